"""Helpers shared by the GPU parity tests: run the HIP library and the CPU oracle on the
same seeded bits and compare element by element."""
import math

import numpy as np
import torch

from oracle import adapm_oracle as O
from paper_2510_09103_amd import workloads as WL

_DT = {"f32": O.F32, "bf16": O.BF16}
_MOM = {"none": O.MOM_NONE, "full": O.MOM_FULL, "lowrank": O.MOM_LOWRANK}
_VM = {"element": O.V_ELEMENT, "rowgroup": O.V_ROWGROUP, "whole": O.V_WHOLE}


def oracle_block(b: WL.BlockSpec) -> O.Block:
    return O.Block(b.rows, b.cols, _DT[b.param_dtype], _DT[b.grad_dtype], _MOM[b.mom], b.rank, _VM[b.v_mode],
                   b.v_group_rows, b.lr_scale, b.weight_decay)


def to_np(t: torch.Tensor) -> np.ndarray:
    """device tensor -> numpy storage array (uint16 bit patterns for bf16)."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def values(a: np.ndarray) -> np.ndarray:
    return O.bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def rel_err_floor(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got-ref| / max(|ref|, RMS(ref)): per element, with a block-RMS floor."""
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    rms = math.sqrt(float(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """distance in representable bf16 values (sign-magnitude -> ordered integers)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def bf16_ulp_of(x: np.ndarray) -> np.ndarray:
    """spacing of bf16 values in the binade of |x|."""
    _, e = np.frexp(np.abs(x))
    return np.ldexp(1.0, np.maximum(e - 8, -133))


# bf16 parameters.  One bf16 ulp is 2^-8 .. 2^-7 relative, above the 2e-3 tolerance, so a result that sits on a
# rounding boundary in fp32 may round the other way on the two sides ("flip"), and since W_{t+1} = W_t - ... a flip
# never heals: the two trajectories of that element stay one ulp OF THE BINADE IT WAS IN THEN apart, which is many
# ulps of its own binade once the element has moved towards zero (lr |u| = 1e-3 per step is 8 ulps of |w| = 0.02, so
# an element crosses a binade in a few steps).  Two checks:
#  * single step from identical parameters (Pair.step): every element at most ONE representable bf16 value apart at
#    its own binade (or within 2e-3 of max(|w|, RMS) where the result cancels towards zero and ulps get tiny), and
#    the fraction of elements that differ at all at most FLIP_PER_STEP (measured: 2e-4 on large blocks, up to 1.1e-3 on
#    blocks of a few thousand elements).  A relative error eps in the update flips a fraction ~ 8 eps of the
#    elements, so this bound holds the update itself to ~2e-4.
#  * free run over N steps (compare_params): the error of an element is a sum of flips, each one ulp of the binade of
#    its time, so it is measured in ulps of the LARGEST magnitude the element has had along the oracle's trajectory
#    (wmax, tracked per element by Pair): k = |got - ref| / ulp(wmax).  Every element: k <= MAX_FLIPS_FREE or within
#    2e-3 max(|w|, RMS).  Fractions: elements that differ at all <= N * FLIP_PER_STEP; elements with k > 1.5 (two or
#    more flips) <= (N * FLIP_PER_STEP)^2 (both with a Poisson margin for small blocks).  Measured over the
#    configurations' own 20 - 100 steps: 3e-4 .. 7e-3 of the elements differ, 1e-7 .. 2e-5 have k > 1.5, and the
#    largest k is 4.0 (one element in 4 M), so the cap of 5 is never met by chance (five moves one way: (N p)^5 / 5!).
#  The flip rate follows the state error: with the state within tau of the oracle's, the update differs by about tau
#  relative and 8 tau of the elements flip, so runs held to a wider state tolerance (long runs on the MFMA path, whose
#  state drifts) get flip_per_step = max(FLIP_PER_STEP, 10 tau) (Pair.flip_per_step, set by the tests' run()).
FLIP_PER_STEP = 1.5e-3
MAX_FLIPS_FREE = 5
DEBUG_STATS = bool(int(__import__("os").environ.get("ADAPM_PARITY_STATS", "0")))


def poisson_limit(expected_fraction: float, n: int) -> float:
    """upper limit for an observed fraction over n elements whose expectation is at most expected_fraction."""
    mean = expected_fraction * n
    return min(1.0, (mean + 4.0 * math.sqrt(mean) + 1.0) / max(n, 1))


def compare_params(got: np.ndarray, ref: np.ndarray, tol: float, tol_bf16: float = 2e-3, wmax: np.ndarray = None):
    """fp32 params: |got-ref| <= tol * max(|ref|, RMS(ref)).  bf16 params: see above (wmax: largest |w| of every
    element along the oracle's trajectory; None: the larger of the two present magnitudes).
    Returns (ok, worst relative error of the offenders, fraction not bit-equal, fraction two or more flips apart)."""
    if ref.dtype == np.uint16:
        g, r = values(got), values(ref)
        rms = math.sqrt(float(np.mean(r * r))) if r.size else 0.0
        diff = np.abs(g - r)
        rel = diff / np.maximum(np.abs(r), max(rms, 1e-300))
        top = np.maximum(np.abs(g), np.abs(r))
        if wmax is not None:
            top = np.maximum(top, wmax.reshape(-1))
        k = diff / bf16_ulp_of(top)
        if DEBUG_STATS:
            sel = rel > tol_bf16
            print(f"    bf16 free run: n={k.size} differ={np.mean(got != ref):.2e} k>1.5: {np.mean((k > 1.5) & sel):.2e} "
                  f"k>3: {np.mean((k > 3) & sel):.2e} k>6: {np.mean((k > 6) & sel):.2e} max k={float(k[sel].max()) if sel.any() else 0:.1f} "
                  f"rms diff/rms={math.sqrt(float(np.mean(diff * diff))) / max(rms, 1e-300):.2e}", flush=True)
        fine = (k <= MAX_FLIPS_FREE) | (rel <= tol_bf16)
        bad = rel[~fine]
        far = (k > 1.5) & (rel > tol_bf16)
        return (bool(np.all(fine)), float(bad.max()) if bad.size else 0.0, float(np.mean(got != ref)) if ref.size else 0.0,
                float(np.mean(far)) if ref.size else 0.0)
    e = rel_err_floor(got, ref)
    return e <= tol, e, 0.0, 0.0


class Pair:
    """The library and the oracle stepping side by side on one workload."""

    def __init__(self, wl: WL.Workload, hp_kwargs=None, device="cuda:0", grad_scale=1.0, grad_clip=None):
        from paper_2510_09103_amd.optimizer import AdaPM, make_hparams
        hp_kwargs = dict(hp_kwargs or {})
        self.wl = wl
        base = dict(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K)
        base.update(hp_kwargs)
        self.hp_c = make_hparams(**base)
        ok = {k: v for k, v in base.items() if k != "contraction"}
        self.hp_o = O.HParams(**ok) if "seed" in ok else O.HParams(**ok, seed=0x5EED)
        self.grad_clip = grad_clip
        self.opt = AdaPM(wl.blocks, self.hp_c, device=device, grad_clip=grad_clip or 0.0)
        # the workspace is scratch: poison it (every byte 0xFF = NaN in bf16, fp32 and fp64) so that anything read
        # before it was written in the same step shows up whatever the allocator handed out
        self.opt.workspace.fill_(255)
        self.blocks_o = [oracle_block(b) for b in wl.blocks]
        self.state_o = O.init_state(self.blocks_o, self.hp_o)
        self.params = WL.initial_params(wl, device=device)
        self.W_o = [to_np(p) for p in self.params]
        self.stream = WL.GradientStream(wl, device=device, scale=grad_scale)
        self.t = 0
        self.single_step_flips = 0.0
        self.flip_per_step = FLIP_PER_STEP
        # largest magnitude every bf16 parameter has had along the oracle's trajectory (see compare_params)
        self.wmax = {i: np.abs(values(w).reshape(-1)) for i, w in enumerate(self.W_o) if wl.blocks[i].param_dtype == "bf16"}

    def step(self, lr=None, oracle_only=None):
        self.t += 1
        lr = self.wl.lr if lr is None else lr
        grads = self.stream.next()
        W_before = [to_np(p) for p in self.params]          # the library's own parameters before the step
        self.opt.step(self.params, grads, self.t, lr)
        G_o = [to_np(g) for g in grads]
        self.W_o, self.state_o, forced = O.step(self.blocks_o, self.hp_o, self.W_o, G_o, self.state_o, self.t, lr,
                                                only=oracle_only, Ws_alt=W_before, grad_clip=self.grad_clip)
        if self.grad_clip:
            # the norm and the factor the library derived on the device against the oracle's
            norm, scale = self.opt.last_grad_norm()
            s_o, n_o = O.global_grad_scale(self.blocks_o, G_o, self.grad_clip)
            assert abs(norm - n_o) <= 1e-6 * n_o and abs(scale - s_o) <= 1e-6 * s_o, (norm, n_o, scale, s_o)
        # single-step check from identical parameters: bf16 results at most ONE representable value apart, and
        # only a bounded fraction of them apart at all
        idx = range(len(self.wl.blocks)) if oracle_only is None else oracle_only
        for i in idx:
            if self.wl.blocks[i].param_dtype == "bf16":
                got, ref = to_np(self.params[i]).reshape(-1), forced[i].reshape(-1)
                d = bf16_ulp_distance(got, ref)
                if int(d.max()) > 1:      # results that cancel towards zero have tiny ulps: fall back to the tolerance
                    r = values(ref)
                    rel = np.abs(values(got) - r) / np.maximum(np.abs(r), math.sqrt(float(np.mean(r * r))))
                    worst = float(rel[d > 1].max())
                    assert worst <= 2e-3, (f"step {self.t} block {i} ({self.wl.blocks[i].name}): {int(d.max())} bf16 ulps "
                                           f"and {worst:.2e} relative apart after one step")
                flips = float(np.mean(d != 0))
                limit = poisson_limit(self.flip_per_step, d.size)
                assert flips <= limit, (f"step {self.t} block {i} ({self.wl.blocks[i].name}): {flips:.2e} of the bf16 "
                                        f"parameters differ after ONE step from identical values (bound {limit:.2e})")
                self.single_step_flips = max(self.single_step_flips, flips)
                self.wmax[i] = np.maximum(self.wmax[i], np.abs(values(self.W_o[i]).reshape(-1)))
        return grads

    def compare(self, tol_state, tol_param, only=None, products_only=False):
        """returns a report dict; raises AssertionError with the worst offender."""
        torch.cuda.synchronize()
        worst = {"state": 0.0, "param": 0.0, "flip_frac_bf16": 0.0, "far_frac_bf16": 0.0,
                 "flip_frac_single_step": self.single_step_flips}
        idx = range(len(self.wl.blocks)) if only is None else only
        for i in idx:
            b = self.wl.blocks[i]
            sv = {k: v.cpu().numpy() for k, v in self.opt.state_view(i).items()}
            so = self.state_o[i]
            for key in ("m", "v"):
                if key in so:
                    e = rel_err_floor(sv[key].reshape(-1), so[key].reshape(-1))
                    worst["state"] = max(worst["state"], e)
                    assert e <= tol_state, f"block {i} ({b.name}) state {key}: rel err {e:.3e} > {tol_state}"
            if "L" in so:
                prod_g = sv["L"].astype(np.float64) @ sv["R"].astype(np.float64)
                prod_o = so["L"].astype(np.float64) @ so["R"].astype(np.float64)
                e = rel_err_floor(prod_g, prod_o)
                worst["state"] = max(worst["state"], e)
                assert e <= tol_state, f"block {i} ({b.name}) product LR: rel err {e:.3e} > {tol_state}"
                if not products_only:
                    for key in ("L", "R"):
                        e = rel_err_floor(sv[key], so[key])
                        worst["state"] = max(worst["state"], e)
                        assert e <= tol_state, f"block {i} ({b.name}) factor {key}: rel err {e:.3e} > {tol_state}"
            ok, e, flips, far = compare_params(to_np(self.params[i]).reshape(-1), self.W_o[i].reshape(-1), tol_param,
                                               wmax=self.wmax.get(i))
            worst["param"] = max(worst["param"], e)
            assert ok, (f"block {i} ({b.name}) params: rel err {e:.3e} > {tol_param}"
                        + (f" and more than {MAX_FLIPS_FREE} flips apart" if b.param_dtype == "bf16" else ""))
            if b.param_dtype == "bf16":
                # flip statistics over bf16 blocks only (fp32 parameters differ in their last bits as a matter of course)
                n, q = b.rows * b.cols, min(1.0, self.t * self.flip_per_step)
                worst["flip_frac_bf16"] = max(worst["flip_frac_bf16"], flips)
                worst["far_frac_bf16"] = max(worst["far_frac_bf16"], far)
                assert flips <= poisson_limit(q, n), (f"block {i} ({b.name}): {flips:.2e} of the bf16 parameters differ "
                                                      f"after {self.t} steps (bound {poisson_limit(q, n):.2e})")
                assert far <= poisson_limit(q * q, n), (f"block {i} ({b.name}): {far:.2e} of the bf16 parameters are two or "
                                                        f"more flips apart after {self.t} steps (bound {poisson_limit(q * q, n):.2e})")
        return worst
