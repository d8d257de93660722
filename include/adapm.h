/*
 * adapm.h - C ABI of the AdaPM optimizer step for AMD MI355X (gfx950).
 *
 * The library applies, to every parameter block of a model, one step of the
 * paper's update (Alg. 1 "Low Rank Update with Correction"): full momentum
 * (eq. 5), no momentum (Sec. 4.1 regime 1) or bias-corrected low-rank momentum
 * (eq. 2-4, tracked by the gradient-descent solver of Alg. 2 / App. B), a
 * per-element or blockwise second moment (Alg. 1 "v_t"; blockwise mean as in the
 * Adam-mini combination of Sec. 5.1.3), and the clipped update with decoupled
 * weight decay (Alg. 1 last line).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; every other
 *    pointer is HOST memory.  The library owns only the context object (a host
 *    plan plus small device-side tables, released by adapm_destroy).
 *  - A block is one parameter tensor, row-major rows x cols, rows = output units;
 *    1-D tensors use cols = 1.  Block base pointers must be 16-byte aligned.
 *  - adapm_step is asynchronous on the given HIP stream and updates params and state in
 *    place; grads are read-only.  It allocates nothing once adapm_state_init has run on
 *    the context (which places the launch plan on the device), unless per-launch timing
 *    is on, and it never waits for the device: the pointer tables live on the device in a
 *    few slots keyed by their contents (a caller that rotates up to four sets of tensors
 *    uploads each once; a new set is copied on the step's stream).  Issue the steps of one
 *    context on one stream, or order the streams yourself.
 *  - Functions return ADAPM_OK (0) or a negative status; nothing aborts or throws.
 *    adapm_last_error() gives a thread-local message for the last failure.
 *  - bf16 tensors are IEEE-like bfloat16 bit patterns; stores round to nearest even.
 */
#ifndef ADAPM_H
#define ADAPM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ADAPM_OK = 0,
  ADAPM_EINVAL = -1,   /* bad argument / table entry */
  ADAPM_ENOMEM = -2,   /* host or device allocation of the context failed */
  ADAPM_EHIP = -3,     /* a HIP runtime call failed */
  ADAPM_ESTATE = -4    /* call order / step number inconsistent */
} adapm_status_t;

typedef enum { ADAPM_F32 = 0, ADAPM_BF16 = 1 } adapm_dtype_t;

/* Momentum regime of a block (Sec. 4.1): none / full (eq. 5) / low-rank (Alg. 1). */
typedef enum { ADAPM_MOM_NONE = 0, ADAPM_MOM_FULL = 1, ADAPM_MOM_LOWRANK = 2 } adapm_mom_t;

/* Granularity of the second moment: per element (Alg. 1), one value per group of
 * v_group_rows consecutive rows, or one value for the whole block (Sec. 5.1.3). */
typedef enum { ADAPM_V_ELEMENT = 0, ADAPM_V_ROWGROUP = 1, ADAPM_V_WHOLE = 2 } adapm_vmode_t;

/* Arithmetic of the low-rank contractions (G R^T, L^T G, Gram matrices, L R):
 *  F64     - operands exact, fp64 accumulation on the vector ALUs;
 *  BF16X2  - bf16 MFMA with fp32 accumulation, every fp32 factor operand carried
 *            as a (hi, lo) pair of bf16 values (relative operand error 2^-17);
 *            requires bf16 gradients.  Implemented for rank <= 128 (a block runs in
 *            the kernels of the next rank class 32 / 64 / 128, its factors padded
 *            with zeros on chip) and cols >= 8; any other block silently uses F64;
 *  AUTO    - per block: F64 when the block's parameters are fp32, else BF16X2. */
typedef enum { ADAPM_CONTRACT_AUTO = 0, ADAPM_CONTRACT_F64 = 1, ADAPM_CONTRACT_BF16X2 = 2 } adapm_contract_t;

typedef struct {
  int64_t rows, cols;
  int32_t param_dtype, grad_dtype; /* adapm_dtype_t */
  int32_t mom_mode;                /* adapm_mom_t */
  int32_t rank;                    /* LOWRANK only: 1 <= rank <= min(rows, cols); cols >= 2 */
  int32_t v_mode;                  /* adapm_vmode_t */
  int32_t v_group_rows;            /* ROWGROUP: rows % v_group_rows == 0 */
  float lr_scale;                  /* 1.0; the paper uses 0.75 for no-momentum blocks (Sec. 5.1) */
  float weight_decay;              /* lambda of Alg. 1 for this block */
} adapm_block_t;

typedef struct {
  float beta1, beta2, eps;    /* 0.9, 0.95, 1e-8 (Sec. 5.1) */
  float clip;                 /* element-wise clamp of Alg. 1's last line; 1.0; +inf disables */
  int32_t adam_debias;        /* 0 = Alg. 1 as printed; 1 = divide by (1-beta^t) (Adam comparison only) */
  int32_t refresh_iters_K;    /* iterations of Alg. 2; 5 (App. B) */
  int32_t refresh_period_T;   /* 1 = Alg. 2 every step (Alg. 1 verbatim).  T > 1: Alg. 2 on steps with
                                 (step-1) % T == 0, followed by a product-preserving orthonormalisation
                                 of R; on other steps L is the least-squares fit with R held.  A block
                                 whose R R^T is not positive definite at that point (R has lost rank)
                                 keeps its (L, R) as Alg. 2 left them. */
  int32_t bias_correction;    /* 1 = eq. 4; 0 = ablation of Sec. 5.1.2 (use L_t R_t as the momentum) */
  int32_t contraction;        /* adapm_contract_t */
  int32_t refresh_normalise;  /* 0 = Alg. 2 as printed.  1 (an option beyond the paper): every iteration of Alg. 2
                                 divides its step size by max(||R R^T||_F, ||L^T L||_F), which makes the
                                 iteration invariant under a rescaling of the gradients (as printed it
                                 diverges for large and stalls for small gradients) */
  uint64_t seed;              /* seeded start R_0 of the low-rank factors; 0 = literal all-zero start (the factors then
                                 stay zero for ever; only with refresh_period_T = 1, else ADAPM_EINVAL) */
} adapm_hparams_t;

typedef struct adapm_ctx adapm_ctx;

/* Validate the table and hyper-parameters, fix the state / workspace layout and build
 * the launch plan on the current HIP device.  table[0..nblocks) and hp are read during
 * the call only.  On failure *out is NULL. */
adapm_status_t adapm_init(adapm_ctx** out, const adapm_block_t* table, int64_t nblocks,
                          const adapm_hparams_t* hp);

/* Size of the caller-allocated optimizer state: per block, in table order,
 * [L (rows x rank) | R (rank x cols)] or [m (rows x cols)] or nothing, then v;
 * fp32, each sub-buffer 256-byte aligned (Alg. 1, initialisation).  0 if ctx is NULL. */
size_t adapm_state_bytes(const adapm_ctx* ctx);

/* Size of the caller-allocated scratch buffer used inside adapm_step (previous
 * factors, thin products, Gram matrices, partial sums).  With refresh_period_T > 1 the
 * library also keeps bf16 copies of R there between two runs of Alg. 2: pass the same,
 * unmodified buffer on consecutive steps (a different workspace or state pointer is detected
 * and the copies are rebuilt from that state; overwriting the contents of either buffer
 * between steps is not, see adapm_state_loaded). */
size_t adapm_workspace_bytes(const adapm_ctx* ctx);

/* Byte offsets into the state buffer of block `block`'s sub-buffers; an absent
 * sub-buffer reports (size_t)-1.  Any of L, R, m, v may be NULL. */
adapm_status_t adapm_state_offsets(const adapm_ctx* ctx, int64_t block, size_t* L, size_t* R,
                                   size_t* m, size_t* v);

/* Zero the state and write the seeded R_0 (Alg. 1, initialisation, with L_0 R_0 = 0).
 * Asynchronous on `stream` (a hipStream_t, or NULL for the default stream). */
adapm_status_t adapm_state_init(adapm_ctx* ctx, void* state_dev, void* stream);

/* Tell the library that the caller has overwritten the state buffer (e.g. restored a
 * checkpoint into it): anything derived from the old contents is dropped, and the state is
 * taken to come from a run with the same hyper-parameters (with refresh_period_T > 1: R with
 * orthonormal rows).  Not needed after adapm_state_init. */
adapm_status_t adapm_state_loaded(adapm_ctx* ctx);

/* One optimizer step (Alg. 1) over all blocks.
 *  params_dev / grads_dev: HOST arrays of nblocks DEVICE pointers (table order);
 *  state_dev: adapm_state_bytes() bytes; workspace_dev: adapm_workspace_bytes() bytes
 *  (may be NULL if that size is 0); step: 1-based iteration count t; lr: eta_t.
 * Checks step >= 1, non-null and 16-byte aligned pointers; everything else was
 * validated at init.  With refresh_period_T > 1, a step that holds R on a state whose R has
 * not been orthonormalised (no step that runs Alg. 2 since adapm_state_init, and no
 * adapm_state_loaded) is ADAPM_ESTATE. */
adapm_status_t adapm_step(adapm_ctx* ctx, void* const* params_dev, const void* const* grads_dev,
                          void* state_dev, void* workspace_dev, int64_t step, float lr, void* stream);

/* adapm_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same step with the library's OWN scratch buffer in place of
 * workspace_dev, a fixed array in device memory of adapm_static_scratch_bytes() bytes (64 MiB) that every GPU
 * the library runs on holds until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * event creation): the context must have been set up by adapm_state_init beforehand (else ADAPM_ESTATE) and
 * per-launch timing must be off.  A table whose adapm_workspace_bytes() exceeds the array is ADAPM_EINVAL.
 * All contexts on a GPU share that GPU's array, which keeps whatever the last call left there: the library
 * rebuilds what a context keeps in scratch between steps when another context has used the array in the
 * meantime, and nothing in it is expected to start at zero; calls that overlap in time on one GPU (different
 * streams, different host threads) race on it and are not allowed.  Everything else as adapm_step. */
adapm_status_t adapm_step_static(adapm_ctx* ctx, void* const* params_dev, const void* const* grads_dev,
                                 void* state_dev, int64_t step, float lr, void* stream);

/* Size of the library's own scratch array (see adapm_step_static). */
size_t adapm_static_scratch_bytes(void);

/* Global gradient-norm clipping of the paper's pre-training runs (Sec. 5.1, set-ups: threshold 1.0),
 * folded into the step.  After adapm_set_grad_clip(ctx, c) with c > 0, every adapm_step first sums the
 * squares of all gradients of the table on the device (fixed order, fp64 partial sums), derives
 *     factor = min(1, c / (||G||_2 + 1e-6))
 * there, and uses factor * G wherever the method uses G (second moment, momentum, Alg. 2, update); the
 * caller's gradients are not modified and nothing is read back.  c <= 0 or +inf switches it off (the
 * default); NaN is ADAPM_EINVAL.  Costs one extra pass over the gradients. */
adapm_status_t adapm_set_grad_clip(adapm_ctx* ctx, float max_norm);

/* Norm and factor of the last clipped adapm_step that used workspace_dev (device pointer; NULL: the
 * library's own scratch array, after adapm_step_static): copies two floats to the host and synchronises
 * `stream`.  Either output may be NULL. */
adapm_status_t adapm_last_grad_norm(adapm_ctx* ctx, const void* workspace_dev, void* stream, float* norm, float* scale);

/* Learning-rate schedule of the same runs (Sec. 5.1, set-ups: cosine decay with warm-up), a host helper
 * for the `lr` argument of adapm_step: linear from 0 to peak_lr over warmup_steps, half a cosine down to
 * min_lr at total_steps, min_lr afterwards.  step counts from 1. */
float adapm_lr_cosine_warmup(int64_t step, float peak_lr, float min_lr, int64_t warmup_steps, int64_t total_steps);

/* Arithmetic the planner chose for the contractions of a block (see adapm_contract_t):
 * ADAPM_CONTRACT_F64 or ADAPM_CONTRACT_BF16X2 for a low-rank block, -1 for a block without
 * low-rank momentum or an index out of range. */
int32_t adapm_block_contraction(const adapm_ctx* ctx, int64_t block);

/* Number of kernel launches the last adapm_step enqueued (0 before the first). */
int64_t adapm_last_launch_count(const adapm_ctx* ctx);

/* Compulsory HBM bytes of one step over the table: every input read once and every
 * output written once in its storage type.  refresh_step != 0 counts a step that runs
 * Alg. 2; 0 counts a step with R held (T > 1 only). */
double adapm_algorithmic_bytes(const adapm_ctx* ctx, int32_t refresh_step);

/* Multiply-add work of the low-rank contractions of one step, in flop (2 per multiply-add),
 * counted once per mathematical product (operand splitting not counted). */
double adapm_algorithmic_flops(const adapm_ctx* ctx, int32_t refresh_step);

/* Optional per-launch timing for benchmarks.  While enabled, adapm_step brackets every kernel
 * launch with a pair of HIP events on the caller's stream (this serialises nothing but adds two
 * event records per launch).  For callers that want the duration of each kernel class without an
 * external profiler. */
adapm_status_t adapm_profile_enable(adapm_ctx* ctx, int32_t on);

/* After the caller has synchronised the stream: entry `index` of the per-kernel-class totals
 * accumulated since the last read with index 0 (which folds and clears the pending records).
 * name receives a NUL-terminated label (at most name_cap bytes), total_ms the summed duration,
 * launches the number of launches.  Returns the number of entries. */
int64_t adapm_profile_read(adapm_ctx* ctx, int64_t index, char* name, size_t name_cap, double* total_ms,
                           int64_t* launches);

const char* adapm_last_error(void);

void adapm_destroy(adapm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* ADAPM_H */
