"""Plain CPU oracle of one AdaPM optimizer step, written from the paper.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

What it follows
---------------
* Alg. 1 ("Low Rank Update with Correction"): momentum accumulate, low-rank
  tracking (eq. 2), one-step residual (eq. 3), second moment, bias correction
  (eq. 4), clipped update with decoupled decay.
* Alg. 2 / App. B: K gradient-descent iterations on (L, R), warm-started,
  step sizes eta_k = 0.5 (1 + cos(pi k / K)), k = 1..K.
* eq. 5: the full momentum m^f (blocks in the "full momentum" regime, Sec. 4.1).
* Sec. 4.1 regime (1): blocks with no momentum use the raw gradient.
* Related-work definition of the blockwise second moment (one value per group
  = mean of the per-element statistic over the group), Sec. 5.1.3.

Arithmetic is fp64.  Stored state (L, R, m, v) is rounded to fp32 at the end of
each step; parameters are rounded (round-to-nearest-even, straight from fp64) to
their storage type.  bf16 tensors travel as uint16 bit patterns.

Readings taken where the paper is silent or inconsistent (each is listed in the
design notes of the repository):
* cold start: L_0 = 0 and R_0 = a seeded uniform sketch (so L_0 R_0 = 0 as
  the initialisation of Alg. 1 and the proof of Thm. 2 need, but Alg. 2 can leave zero);
  seed = 0 gives the literal all-zero start.
* Alg. 2 computes both gradients from the same (L, R) before either update.
* clip(., 1) is an element-wise clamp to [-clip, clip].
* lambda x_t is lambda W_t (pre-update W), inside the eta_t bracket.
* global gradient-norm clipping (Sec. 5.1 set-ups) uses scale = min(1, c / (norm + 1e-6)).
* "update frequency T": T = 1 is Alg. 1 verbatim.  For T > 1 Alg. 2 runs on
  steps with (t-1) mod T == 0 and is followed by a product-preserving re-gauge
  (R R^T = C C^T, R <- C^-1 R, L <- L C); on the other steps the arg min
  of Alg. 1 is taken over L with R held, i.e. the least-squares solution.

Parity pins for every function here live in tests/test_oracle_pins.py.  The
T > 1 step is a reading, pinned only by the normal equations ("parity unpinned"
by the paper itself).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

# --- enums (same numeric values as the C header, typed here independently) ---
F32, BF16 = 0, 1
MOM_NONE, MOM_FULL, MOM_LOWRANK = 0, 1, 2
V_ELEMENT, V_ROWGROUP, V_WHOLE = 0, 1, 2


@dataclass
class Block:
    """One parameter tensor, row-major rows x cols (1-D tensors: cols = 1)."""
    rows: int
    cols: int
    param_dtype: int = F32
    grad_dtype: int = F32
    mom_mode: int = MOM_FULL
    rank: int = 0
    v_mode: int = V_ELEMENT
    v_group_rows: int = 1
    lr_scale: float = 1.0
    weight_decay: float = 0.0


@dataclass
class HParams:
    beta1: float = 0.9          # Sec. 5.1 setups
    beta2: float = 0.95
    eps: float = 1e-8
    clip: float = 1.0           # Alg. 1 last line; inf disables
    adam_debias: int = 0        # Alg. 1 has none; 1 only for the Adam pin
    K: int = 5                  # App. B
    T: int = 1                  # 1 = Alg. 1 verbatim
    bias_correction: int = 1    # eq. 4; 0 = ablation of Sec. 5.1.2
    normalise: int = 0          # 1 = scale-normalised step sizes in Alg. 2 (an option beyond the paper)
    seed: int = 0x5EED


# ----------------------------------------------------------------------------
# storage types
# ----------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp64, exact."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bit patterns, round-to-nearest-even in ONE rounding.

    bf16 keeps 8 significant bits; for |x| in [2^(e-1), 2^e) the spacing is
    2^(e-8) (2^-133 in the subnormal range).  x / spacing is exact, np.rint
    rounds ties to even.
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    q = np.ldexp(1.0, np.maximum(e - 8, -133))
    y = np.rint(x / q) * q
    with np.errstate(over="ignore"):
        f = y.astype(np.float32)        # exact: y has <= 8 significant bits
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def load(a: np.ndarray, dtype: int) -> np.ndarray:
    """storage array -> fp64 values (exact)."""
    if dtype == BF16:
        return bf16_bits_to_f64(a)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def store(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp64 values -> storage array, RNE."""
    if dtype == BF16:
        return f64_to_bf16_bits(x)
    return np.asarray(x, dtype=np.float64).astype(np.float32)


# ----------------------------------------------------------------------------
# cold start (reading of the initialisation of Alg. 1)
# ----------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def _mix64(z: int) -> int:
    """The 64-bit finaliser of the SplitMix64 generator (Steele et al. 2014)."""
    z = (z + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = z + np.uint64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def sketch_R0(seed: int, block_index: int, r: int, n: int) -> np.ndarray:
    """Seeded start R_0 (r x n, fp32): counter-based, uniform, sigma_max ~ 1.

    key  = mix(seed XOR mix(block_index));  h_i = mix(key + i), i = a*n + j
    k_i  = (h_i >> 40) - 2^23            (an integer in [-2^23, 2^23))
    R_0  = fp32(k_i) * fp32( sqrt(3) / (sqrt(n) + sqrt(r)) * 2^-23 )
    The standard deviation is 1 / (sqrt(n) + sqrt(r)).  seed == 0 -> zeros.
    """
    if seed == 0:
        return np.zeros((r, n), dtype=np.float32)
    key = _mix64((seed & _M64) ^ _mix64(block_index & _M64))
    with np.errstate(over="ignore"):
        idx = np.arange(r * n, dtype=np.uint64) + np.uint64(key)
        h = _mix64_np(idx)
    k = (h >> np.uint64(40)).astype(np.int64) - (1 << 23)
    amp = np.float32(math.sqrt(3.0) / (math.sqrt(float(n)) + math.sqrt(float(r))) * 2.0 ** -23)
    return (k.astype(np.float32) * amp).reshape(r, n)


def num_v(blk: Block) -> int:
    if blk.v_mode == V_ELEMENT:
        return blk.rows * blk.cols
    if blk.v_mode == V_ROWGROUP:
        return blk.rows // blk.v_group_rows
    return 1


def init_state(blocks: List[Block], hp: HParams, dtype=np.float32) -> List[Dict[str, np.ndarray]]:
    """Initialisation of Alg. 1 with the cold-start reading above; m^f_0 = 0 (eq. 5)."""
    out = []
    for i, b in enumerate(blocks):
        st: Dict[str, np.ndarray] = {"v": np.zeros(num_v(b), dtype=dtype)}
        if b.mom_mode == MOM_FULL:
            st["m"] = np.zeros((b.rows, b.cols), dtype=dtype)
        elif b.mom_mode == MOM_LOWRANK:
            st["L"] = np.zeros((b.rows, b.rank), dtype=dtype)
            st["R"] = sketch_R0(hp.seed, i, b.rank, b.cols).astype(dtype)
        out.append(st)
    return out


# ----------------------------------------------------------------------------
# Alg. 2 and its alternatives
# ----------------------------------------------------------------------------
def gd_step_sizes(K: int) -> List[float]:
    """App. B: eta_k = 0.5 (1 + cos(pi k / K)), k = 1..K (the last one is 0)."""
    return [0.5 * (1.0 + math.cos(math.pi * k / K)) for k in range(1, K + 1)]


def refresh_gd(M: np.ndarray, L: np.ndarray, R: np.ndarray, K: int, normalise: bool = False):
    """Alg. 2: K simultaneous gradient steps on l(L,R) with the printed gradients
    dl/dL = (L R - M) R^T,  dl/dR = L^T (L R - M).

    normalise (an option beyond the paper; Alg. 2 as printed takes eta_k as is, which diverges once the
    gradients' largest singular value passes a few units and stalls when it is small): every iteration
    divides its step size by nu = max(||R R^T||_F, ||L^T L||_F), an upper bound of the curvature of l in
    either factor, so that the iteration is invariant under (L, R, M) -> (sqrt(c) L, sqrt(c) R, c M)."""
    L = L.copy()
    R = R.copy()
    for eta in gd_step_sizes(K):
        if normalise:
            nu = max(float(np.linalg.norm(R @ R.T)), float(np.linalg.norm(L.T @ L)))
            if nu > 0.0:
                eta = eta / nu
        E = L @ R - M
        dL = E @ R.T
        dR = L.T @ E
        L = L - eta * dL
        R = R - eta * dR
    return L, R


def refresh_exact(M: np.ndarray, r: int):
    """An exact minimiser of eq. 2 (Eckart-Young): truncated SVD, balanced split."""
    U, s, Vt = np.linalg.svd(M, full_matrices=False)
    rs = np.sqrt(s[:r])
    return U[:, :r] * rs, rs[:, None] * Vt[:r, :]


def regauge(L: np.ndarray, R: np.ndarray):
    """Product-preserving change of factors: R R^T = C C^T (C lower, positive
    diagonal), R <- C^-1 R (orthonormal rows), L <- L C."""
    C = np.linalg.cholesky(R @ R.T)
    return L @ C, np.linalg.solve(C, R)


def lstsq_L(M: np.ndarray, R: np.ndarray) -> np.ndarray:
    """arg-min over L of ||L R - M||_F^2 with R held: L = M R^T (R R^T)^-1."""
    return np.linalg.solve(R @ R.T, R @ M.T).T


def is_refresh_step(t: int, T: int) -> bool:
    return T <= 1 or (t - 1) % T == 0


# ----------------------------------------------------------------------------
# the step
# ----------------------------------------------------------------------------
def second_moment(blk: Block, hp: HParams, g: np.ndarray, v_prev: np.ndarray):
    """v_t = beta2 v_{t-1} + (1-beta2) * (mean over the group of g^2).
    Returns (v_t as stored shape, v_t broadcast to rows x cols)."""
    g2 = g * g
    if blk.v_mode == V_ELEMENT:
        v = hp.beta2 * v_prev.reshape(blk.rows, blk.cols) + (1.0 - hp.beta2) * g2
        return v.reshape(-1), v
    if blk.v_mode == V_ROWGROUP:
        gr = blk.v_group_rows
        ng = blk.rows // gr
        mean = g2.reshape(ng, gr * blk.cols).mean(axis=1)
        v = hp.beta2 * v_prev + (1.0 - hp.beta2) * mean
        return v, np.repeat(v, gr)[:, None] * np.ones((1, blk.cols))
    mean = g2.mean()
    v = hp.beta2 * v_prev + (1.0 - hp.beta2) * mean
    return v, np.full((blk.rows, blk.cols), v[0])


def step_block(blk: Block, hp: HParams, W: np.ndarray, G: np.ndarray,
               st: Dict[str, np.ndarray], t: int, lr: float,
               refresh: str = "GD", state_dtype=np.float32,
               want_aux: bool = False, W_alt: Optional[np.ndarray] = None, g_scale: float = 1.0):
    """One optimizer step on one block.  t is 1-based.

    W, G: storage arrays (float32, or uint16 bit patterns for bf16), any shape
    with rows*cols elements.  Returns (W_new storage, new state dict, aux).
    W_alt: a second parameter tensor pushed through the same last line (W enters Alg. 1
    nowhere else); its result is returned as aux["W_alt_new"].
    g_scale: factor of the global gradient clipping; the method then sees g_scale * G."""
    m_, n_ = blk.rows, blk.cols
    g = load(G, blk.grad_dtype).reshape(m_, n_) * g_scale
    w = load(W, blk.param_dtype).reshape(m_, n_)
    b1, b2 = hp.beta1, hp.beta2
    new: Dict[str, np.ndarray] = {}
    aux: Dict[str, np.ndarray] = {}

    # second moment (Alg. 1, "standard second-order momentum update"; blockwise mean)
    v_store, v_full = second_moment(blk, hp, g, st["v"].astype(np.float64))
    new["v"] = v_store.astype(state_dtype)

    # momentum by regime (Sec. 4.1)
    if blk.mom_mode == MOM_NONE:
        mc = g
    elif blk.mom_mode == MOM_FULL:
        m = (1.0 - b1) * g + b1 * st["m"].astype(np.float64).reshape(m_, n_)   # eq. 5
        new["m"] = m.astype(state_dtype)
        mc = m
    else:
        Lp = st["L"].astype(np.float64)
        Rp = st["R"].astype(np.float64)
        A = Lp @ Rp
        M = (1.0 - b1) * g + b1 * A                      # Alg. 1: m_t
        if is_refresh_step(t, hp.T):
            if refresh == "GD":
                L, R = refresh_gd(M, Lp, Rp, hp.K, normalise=bool(hp.normalise))     # Alg. 2
            elif refresh == "EXACT":
                L, R = refresh_exact(M, blk.rank)
            else:
                raise ValueError(refresh)
            if hp.T > 1:
                L, R = regauge(L, R)
        else:
            L, R = lstsq_L(M, Rp), Rp
        B = L @ R
        res = B - M                                      # eq. 3: r_t
        if hp.bias_correction:
            mc = M - b1 * res / (1.0 - b1)               # eq. 4
        else:
            mc = B
        new["L"] = L.astype(state_dtype)
        new["R"] = R.astype(state_dtype)
        if want_aux:
            aux.update(A=A, M=M, B=B, r=res)

    vv = v_full
    if hp.adam_debias:
        mc = mc / (1.0 - b1 ** t)
        vv = vv / (1.0 - b2 ** t)

    # Alg. 1 last line
    u = mc / (np.sqrt(vv) + hp.eps)
    if math.isfinite(hp.clip):
        u = np.clip(u, -hp.clip, hp.clip)
    w_new = w - (lr * blk.lr_scale) * (u + blk.weight_decay * w)
    if want_aux:
        aux.update(mc=mc, u=u, v_full=v_full, w_new=w_new)
    if W_alt is not None:
        wa = load(W_alt, blk.param_dtype).reshape(m_, n_)
        wa_new = wa - (lr * blk.lr_scale) * (u + blk.weight_decay * wa)
        aux["W_alt_new"] = store(wa_new, blk.param_dtype).reshape(np.shape(W_alt))
    return store(w_new, blk.param_dtype).reshape(np.shape(W)), new, aux


def global_grad_scale(blocks: List[Block], Gs: List[np.ndarray], max_norm: float, eps: float = 1e-6):
    """Global gradient-norm clipping of the paper's pre-training runs (Sec. 5.1, set-ups: "global
    gradient clipping at a threshold of 1.0"): ONE factor for the whole table,
        scale = min(1, max_norm / (||G||_2 + eps)),
    ||G||_2 the Euclidean norm over every entry of every gradient.  The paper prints no formula; this is
    the convention of the training code it builds on (a reading, listed in the design notes).
    Gs are storage arrays (float32, or uint16 bit patterns for bf16).  Returns (scale, norm)."""
    total = 0.0
    for blk, g in zip(blocks, Gs):
        g64 = load(g, blk.grad_dtype)
        total += float(np.sum(g64 * g64))
    norm = math.sqrt(total)
    return min(1.0, float(max_norm) / (norm + eps)), norm


def lr_cosine_warmup(t: int, peak_lr: float, min_lr: float, warmup_steps: int, total_steps: int) -> float:
    """Learning-rate schedule of the paper's pre-training runs (Sec. 5.1, set-ups: cosine decay with
    2000 warm-up steps): linear from 0 to peak_lr over the warm-up, then half a cosine down to min_lr at
    total_steps, constant min_lr afterwards.  t counts steps from 1."""
    if warmup_steps > 0 and t <= warmup_steps:
        return peak_lr * t / warmup_steps
    if t >= total_steps:
        return min_lr
    x = (t - warmup_steps) / (total_steps - warmup_steps)
    return min_lr + 0.5 * (peak_lr - min_lr) * (1.0 + math.cos(math.pi * x))


def step(blocks: List[Block], hp: HParams, Ws: List[np.ndarray], Gs: List[np.ndarray],
         state: List[Dict[str, np.ndarray]], t: int, lr: float, refresh: str = "GD",
         only: Optional[List[int]] = None, Ws_alt: Optional[List[np.ndarray]] = None,
         grad_clip: Optional[float] = None):
    """One step over a block table (blocks are independent; `only` selects a subset).
    With Ws_alt, also returns the alternative parameters after the same update.
    With grad_clip, every gradient of the table is first multiplied by global_grad_scale(Gs, grad_clip)
    (the norm is over ALL gradients handed in, whatever `only` selects)."""
    g_scale = 1.0
    if grad_clip is not None and grad_clip > 0 and math.isfinite(grad_clip):
        g_scale, _ = global_grad_scale(blocks, Gs, grad_clip)
    idx = range(len(blocks)) if only is None else only
    Ws = list(Ws)
    state = list(state)
    alt = list(Ws_alt) if Ws_alt is not None else None
    for i in idx:
        Ws[i], state[i], aux = step_block(blocks[i], hp, Ws[i], Gs[i], state[i], t, lr, refresh,
                                          W_alt=None if alt is None else alt[i], g_scale=g_scale)
        if alt is not None:
            alt[i] = aux["W_alt_new"]
    return (Ws, state) if alt is None else (Ws, state, alt)


def state_bytes_closed_form(blocks: List[Block]) -> int:
    """Optimizer-state size in fp32 with no padding: L, R for low-rank blocks
    (Alg. 1, initialisation), m for full-momentum blocks, one v per group."""
    tot = 0
    for b in blocks:
        if b.mom_mode == MOM_LOWRANK:
            tot += 4 * (b.rows + b.cols) * b.rank
        elif b.mom_mode == MOM_FULL:
            tot += 4 * b.rows * b.cols
        tot += 4 * num_v(b)
    return tot
