"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test is chosen so that a plausible mistake in oracle/adapm_oracle.py (dropped
term, wrong sign, transposed operand, wrong index) fails at least one of them.
None of these tests touches the HIP library.
"""
import math
import os

import numpy as np
import pytest

from oracle import adapm_oracle as O
from oracle import adapm_loops as LO

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def lowrank_grads(m, n, k, steps, seed, p=1.5, sigma=1e-4, rho=0.9, scale=1.0):
    g = rng(seed)
    U, _ = np.linalg.qr(g.standard_normal((m, k)))
    V, _ = np.linalg.qr(g.standard_normal((n, k)))
    s = np.arange(1, k + 1, dtype=np.float64) ** (-p)
    a = np.ones(k)
    out = []
    for _ in range(steps):
        out.append((scale * ((U * (s * a)) @ V.T + sigma * g.standard_normal((m, n)))).astype(np.float32))
        a = rho * a + math.sqrt(1 - rho * rho) * g.standard_normal(k)
    return out


# ---------------------------------------------------------------------------
# storage types and the seeded start
# ---------------------------------------------------------------------------
def test_bf16_rne_matches_library_conversion():
    torch = pytest.importorskip("torch")
    g = rng(0)
    x = np.concatenate([
        g.standard_normal(20000).astype(np.float32),
        (g.standard_normal(2000) * 1e-30).astype(np.float32),
        (g.standard_normal(2000) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38], dtype=np.float32),
    ])
    # exact ties: 8 significant bits + a half-ulp bit set
    ties = (np.arange(256, 512, dtype=np.float64) * 2 + 1) / 512.0
    x = np.concatenate([x, ties.astype(np.float32)])
    ours = O.f64_to_bf16_bits(x.astype(np.float64))
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, lib)
    back = O.bf16_bits_to_f64(ours)
    lib_back = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(back, lib_back)


def test_bf16_single_rounding_from_fp64():
    # 1 + 2^-8 + 2^-40 lies just above a tie: one rounding goes up, rounding through
    # fp32 first (-> exactly the tie 1 + 2^-8) would go to even, i.e. down.
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40])
    assert O.bf16_bits_to_f64(O.f64_to_bf16_bits(x))[0] == 1.0 + 2.0 ** -7


def test_mix64_known_answer():
    # first outputs of the SplitMix64 generator started from state 0 (published test vector)
    assert O._mix64(0) == 0xE220A8397B1DCDAF
    assert int(O._mix64_np(np.array([0], dtype=np.uint64))[0]) == 0xE220A8397B1DCDAF


def test_sketch_R0_statistics_and_determinism():
    r, n = 32, 2048
    R = O.sketch_R0(123, 7, r, n)
    assert R.dtype == np.float32 and R.shape == (r, n)
    assert np.array_equal(R, O.sketch_R0(123, 7, r, n))
    assert not np.array_equal(R, O.sketch_R0(123, 8, r, n))
    assert not np.array_equal(R, O.sketch_R0(124, 7, r, n))
    target = 1.0 / (math.sqrt(n) + math.sqrt(r))
    assert abs(R.std() / target - 1) < 0.02
    assert abs(R.mean()) < 4 * target / math.sqrt(r * n)
    smax = np.linalg.svd(R.astype(np.float64), compute_uv=False)[0]
    assert 0.9 < smax < 1.1
    assert np.all(O.sketch_R0(0, 7, r, n) == 0)


def test_gd_step_sizes_closed_form():
    # cos(pi/5) = (1 + sqrt 5)/4, cos(2 pi/5) = (sqrt 5 - 1)/4; App. B schedule with K = 5
    c1, c2 = (1 + math.sqrt(5)) / 4, (math.sqrt(5) - 1) / 4
    want = [0.5 * (1 + c1), 0.5 * (1 + c2), 0.5 * (1 - c2), 0.5 * (1 - c1), 0.0]
    got = O.gd_step_sizes(5)
    assert np.allclose(got, want, atol=1e-15)
    assert got[-1] < 1e-16 and got[0] == pytest.approx(0.904508, abs=1e-6)


# ---------------------------------------------------------------------------
# P1: every block full momentum + per-element v  ==  Adam
# ---------------------------------------------------------------------------
def _run_full(hp, blk, W0, Gs, lr):
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    W = W0.copy()
    Wt = []
    for t, G in enumerate(Gs, 1):
        Wn, st, _ = O.step_block(blk, hp, W, G, st, t, lr, state_dtype=np.float64, want_aux=True)
        W = Wn
        Wt.append(W.astype(np.float64))
    return W, st, Wt


def test_P1a_unrolled_closed_form_no_debias():
    g = rng(1)
    m_, n_, T = 5, 7, 6
    b1, b2, eps, lam, lr = 0.9, 0.95, 1e-8, 0.1, 1e-2
    hp = O.HParams(beta1=b1, beta2=b2, eps=eps, clip=math.inf)
    blk = O.Block(m_, n_, mom_mode=O.MOM_FULL, weight_decay=lam)
    Gs = [g.standard_normal((m_, n_)).astype(np.float32) for _ in range(T)]
    W0 = g.standard_normal((m_, n_)).astype(np.float32)
    # closed form by direct sums (eq. 5 unrolled; Alg. 1 v_t unrolled)
    W = W0.astype(np.float64)
    for t in range(1, T + 1):
        m = sum((1 - b1) * b1 ** (t - i) * Gs[i - 1].astype(np.float64) for i in range(1, t + 1))
        v = sum((1 - b2) * b2 ** (t - i) * Gs[i - 1].astype(np.float64) ** 2 for i in range(1, t + 1))
        W = W - lr * (m / (np.sqrt(v) + eps) + lam * W)
    # the oracle keeps W in fp32 storage; feed it through fp64 storage instead for an exact check
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    w = W0.astype(np.float64)
    for t in range(1, T + 1):
        _, st, aux = O.step_block(blk, hp, w.astype(np.float32), Gs[t - 1], st, t, lr,
                                  state_dtype=np.float64, want_aux=True)
        # redo the last line from aux with the un-rounded w to avoid fp32 storage
        w = w - lr * (aux["u"] + lam * w)
    assert np.allclose(w, W, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("lam", [0.0, 0.1])
def test_P1b_matches_library_adam_adamw(lam):
    torch = pytest.importorskip("torch")
    g = rng(2)
    m_, n_, T = 6, 5, 8
    b1, b2, eps, lr = 0.9, 0.95, 1e-8, 3e-3
    hp = O.HParams(beta1=b1, beta2=b2, eps=eps, clip=math.inf, adam_debias=1)
    blk = O.Block(m_, n_, mom_mode=O.MOM_FULL, weight_decay=lam)
    Gs = [g.standard_normal((m_, n_)).astype(np.float32) for _ in range(T)]
    W0 = g.standard_normal((m_, n_)).astype(np.float32)
    p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = (torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=lam) if lam
           else torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps))
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    w = W0.astype(np.float64)
    for t in range(1, T + 1):
        p.grad = torch.tensor(Gs[t - 1], dtype=torch.float64)
        opt.step()
        _, st, aux = O.step_block(blk, hp, w.astype(np.float32), Gs[t - 1], st, t, lr,
                                  state_dtype=np.float64, want_aux=True)
        w = w - lr * (aux["u"] + lam * w)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-11, atol=1e-13), t
    # and through fp32 storage the oracle's own W stays within fp32 rounding of it
    W, _, _ = _run_full(hp, blk, W0, Gs, lr)
    assert np.allclose(W, p.detach().numpy(), rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------------------
# P2: an exact full-rank arg-min has zero residual; low-rank == full momentum
# ---------------------------------------------------------------------------
def test_P2_full_rank_exact_zero_residual_equals_full_momentum():
    g = rng(3)
    m_, n_, T = 6, 4, 5
    hp = O.HParams(clip=1.0, seed=11)
    lo = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=min(m_, n_), weight_decay=0.1)
    fu = O.Block(m_, n_, mom_mode=O.MOM_FULL, weight_decay=0.1)
    Gs = [g.standard_normal((m_, n_)).astype(np.float32) for _ in range(T)]
    W0 = g.standard_normal((m_, n_)).astype(np.float32)
    s_lo = O.init_state([lo], hp, dtype=np.float64)[0]
    s_fu = O.init_state([fu], hp, dtype=np.float64)[0]
    Wl, Wf = W0.copy(), W0.copy()
    for t in range(1, T + 1):
        Wl, s_lo, aux = O.step_block(lo, hp, Wl, Gs[t - 1], s_lo, t, 1e-2, refresh="EXACT",
                                     state_dtype=np.float64, want_aux=True)
        Wf, s_fu, _ = O.step_block(fu, hp, Wf, Gs[t - 1], s_fu, t, 1e-2, state_dtype=np.float64)
        assert np.abs(aux["r"]).max() < 1e-13
        assert np.allclose(aux["mc"], s_fu["m"], atol=1e-13)
        assert np.allclose(s_lo["L"] @ s_lo["R"], s_fu["m"], atol=1e-13)
        assert np.array_equal(Wl, Wf) or np.allclose(Wl, Wf, rtol=0, atol=1e-7)


# ---------------------------------------------------------------------------
# P3 / P4 / P7: the correction term, Thm. 2's recursion, frozen factors
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("refresh", ["GD", "EXACT"])
def test_P3_P4_bias_correction_and_thm2_recursion(refresh):
    m_, n_, r, T = 24, 16, 3, 12
    b1 = 0.9
    hp = O.HParams(beta1=b1, seed=5)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    Gs = lowrank_grads(m_, n_, 8, T, seed=4)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    W = np.zeros((m_, n_), dtype=np.float32)
    mf = np.zeros((m_, n_))
    res_hist = []
    for t in range(1, T + 1):
        G = Gs[t - 1].astype(np.float64)
        W, st, aux = O.step_block(blk, hp, W, Gs[t - 1], st, t, 1e-3, refresh=refresh,
                                  state_dtype=np.float64, want_aux=True)
        mf = (1 - b1) * G + b1 * mf                                   # eq. 5
        # eq. 4 two ways
        assert np.allclose(aux["mc"] - aux["M"], -b1 * aux["r"] / (1 - b1), atol=1e-14)
        assert np.allclose(aux["mc"], G + b1 / (1 - b1) * (aux["A"] - aux["B"]), atol=1e-13)
        # proof of Thm. 2: m_t - m^f_t = sum_{i=1}^{t-1} beta1^i r_{t-i}
        want = sum(b1 ** i * res_hist[t - 1 - i] for i in range(1, t)) if t > 1 else 0.0
        assert np.allclose(aux["M"] - mf, want, atol=1e-13), t
        res_hist.append(aux["r"])
    assert np.abs(res_hist[-1]).max() > 1e-6     # the residual is not trivially zero here


def test_P5_beta1_zero_is_clipped_rmsprop():
    m_, n_, r = 10, 12, 2
    hp = O.HParams(beta1=0.0, seed=9)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    Gs = lowrank_grads(m_, n_, 4, 3, seed=6)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    W = np.zeros((m_, n_), dtype=np.float32)
    v = np.zeros((m_, n_))
    for t in range(1, 4):
        G = Gs[t - 1].astype(np.float64)
        W0 = W.astype(np.float64)
        W, st, aux = O.step_block(blk, hp, W, Gs[t - 1], st, t, 1e-2, state_dtype=np.float64, want_aux=True)
        assert np.allclose(aux["mc"], G, atol=1e-15)
        v = 0.95 * v + 0.05 * G * G
        want = W0 - 1e-2 * np.clip(G / (np.sqrt(v) + 1e-8), -1, 1)
        assert np.allclose(aux["w_new"], want, atol=1e-15)


def test_P6_literal_zero_start_never_leaves_zero():
    m_, n_, r = 12, 9, 3
    hp = O.HParams(seed=0)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    Gs = lowrank_grads(m_, n_, 4, 4, seed=7)
    st = O.init_state([blk], hp)[0]
    W = np.zeros((m_, n_), dtype=np.float32)
    for t in range(1, 5):
        W, st, aux = O.step_block(blk, hp, W, Gs[t - 1], st, t, 1e-2, want_aux=True)
        assert np.all(st["L"] == 0) and np.all(st["R"] == 0)
        assert np.allclose(aux["mc"], Gs[t - 1].astype(np.float64), atol=1e-15)


def test_P7_frozen_factors_give_raw_gradient():
    # K = 1 has the single step size eta_1 = 0.5 (1 + cos pi) = 0: factors do not move
    m_, n_, r = 8, 8, 2
    hp = O.HParams(K=1, seed=3)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    g = rng(8)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    st["L"] = g.standard_normal((m_, r))
    G = g.standard_normal((m_, n_)).astype(np.float32)
    _, st2, aux = O.step_block(blk, hp, np.zeros((m_, n_), np.float32), G, st, 1, 1e-2,
                               state_dtype=np.float64, want_aux=True)
    assert np.array_equal(st2["L"], st["L"]) and np.array_equal(st2["R"], st["R"])
    assert np.allclose(aux["mc"], G.astype(np.float64), atol=1e-14)


# ---------------------------------------------------------------------------
# Alg. 2: printed gradients are those of 1/2 ||L R - M||^2; P8 Eckart-Young
# ---------------------------------------------------------------------------
def test_alg2_gradients_by_finite_differences():
    g = rng(10)
    m_, n_, r = 5, 7, 3
    M = g.standard_normal((m_, n_))
    L = g.standard_normal((m_, r))
    R = g.standard_normal((r, n_))
    f = lambda L_, R_: 0.5 * np.sum((L_ @ R_ - M) ** 2)
    # one GD step with K = 2 uses eta_1 = 0.5, eta_2 = 0: recover the gradients from it
    L1, R1 = O.refresh_gd(M, L, R, 2)
    dL, dR = (L - L1) / 0.5, (R - R1) / 0.5
    h = 1e-6
    for (i, k) in [(0, 0), (2, 1), (4, 2)]:
        Lp, Lm = L.copy(), L.copy()
        Lp[i, k] += h
        Lm[i, k] -= h
        assert (f(Lp, R) - f(Lm, R)) / (2 * h) == pytest.approx(dL[i, k], rel=1e-6, abs=1e-7)
    for (k, j) in [(0, 0), (1, 5), (2, 6)]:
        Rp, Rm = R.copy(), R.copy()
        Rp[k, j] += h
        Rm[k, j] -= h
        assert (f(L, Rp) - f(L, Rm)) / (2 * h) == pytest.approx(dR[k, j], rel=1e-6, abs=1e-7)


def test_P8_eckart_young_bound_and_exact_attains_it():
    m_, n_, r = 40, 30, 4
    M = lowrank_grads(m_, n_, 12, 1, seed=11, p=1.0, sigma=1e-3)[0].astype(np.float64)
    s = np.linalg.svd(M, compute_uv=False)
    bound = np.sum(s[r:] ** 2)
    Le, Re = O.refresh_exact(M, r)
    assert np.sum((Le @ Re - M) ** 2) == pytest.approx(bound, rel=1e-10)
    R0 = O.sketch_R0(3, 0, r, n_).astype(np.float64)
    L, R = np.zeros((m_, r)), R0
    prev = np.inf
    for _ in range(400):                       # repeated Alg. 2 calls on a fixed target
        L, R = O.refresh_gd(M, L, R, 5)
        loss = np.sum((L @ R - M) ** 2)
        assert loss >= bound * (1 - 1e-12)
        assert loss <= prev * (1 + 1e-9)
        prev = loss
    assert loss < 1.05 * bound                  # GD approaches the optimum (sigma_1 <= 1)


# ---------------------------------------------------------------------------
# P9: 4 x 4 by hand and by scalar loops
# ---------------------------------------------------------------------------
def _read_golden(name):
    out, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line[1:-1]
                out[cur] = []
            else:
                out[cur].append([float(x) for x in line.split()])
    return {k: np.array(v) for k, v in out.items()}


def test_P9_hand_worked_4x4_rank1():
    gd = _read_golden("hand_4x4_rank1.txt")
    G = gd["G"].astype(np.float32)
    hp = O.HParams(beta1=0.5, beta2=0.75, eps=0.0, clip=2.0, K=2, seed=1)
    blk = O.Block(4, 4, mom_mode=O.MOM_LOWRANK, rank=1, weight_decay=0.5)
    st = {"L": np.zeros((4, 1), np.float32), "R": gd["R0"].astype(np.float32), "v": np.zeros(16, np.float32)}
    W = np.ones((4, 4), np.float32)
    W, st, aux = O.step_block(blk, hp, W, G, st, 1, 0.5, want_aux=True)
    assert np.array_equal(st["L"].ravel(), gd["L1"].ravel())
    assert np.array_equal(st["R"], gd["R1"])
    assert np.array_equal(aux["mc"], gd["mc1"])
    assert np.array_equal(aux["u"], gd["u1"])
    assert np.array_equal(W, gd["W1"])
    W, st, aux = O.step_block(blk, hp, W, G, st, 2, 0.5, want_aux=True)
    assert np.array_equal(st["L"].ravel(), gd["L2"].ravel())
    assert np.array_equal(st["R"], gd["R2"])


@pytest.mark.parametrize("r", [1, 4])
def test_P9_scalar_loops_4x4(r):
    g = rng(12 + r)
    dy = lambda *s: np.round(g.standard_normal(s) * 8) / 8           # dyadic rationals
    G1, G2, W0 = dy(4, 4) + 0.0625, dy(4, 4) + 0.0625, dy(4, 4)
    R0, L0 = dy(r, 4) / 2, np.zeros((4, r))
    b1, b2, eps, clip, lam, lr, K = 0.5, 0.5, 1e-8, 1.0, 0.25, 0.125, 2
    hp = O.HParams(beta1=b1, beta2=b2, eps=eps, clip=clip, K=K, seed=1)
    blk = O.Block(4, 4, mom_mode=O.MOM_LOWRANK, rank=r, weight_decay=lam)
    st = {"L": L0.copy(), "R": R0.copy(), "v": np.zeros(16)}
    W = W0.astype(np.float32)
    Wl, Ll, Rl, vl = W0.tolist(), L0.tolist(), R0.tolist(), np.zeros((4, 4)).tolist()
    for t, G in enumerate([G1, G2], 1):
        W, st, aux = O.step_block(blk, hp, W, G.astype(np.float32), st, t, lr,
                                  state_dtype=np.float64, want_aux=True)
        Wl, Ll, Rl, vl, mcl, resl = LO.lowrank_step(Wl, G.tolist(), Ll, Rl, vl, b1, b2, eps, clip, lam, lr, K)
        assert np.allclose(st["L"], np.array(Ll), rtol=1e-13, atol=1e-15)
        assert np.allclose(st["R"], np.array(Rl), rtol=1e-13, atol=1e-15)
        assert np.allclose(aux["r"], np.array(resl), rtol=1e-12, atol=1e-14)
        assert np.allclose(aux["mc"], np.array(mcl), rtol=1e-12, atol=1e-14)
        assert np.allclose(st["v"].reshape(4, 4), np.array(vl), rtol=1e-14)
        assert np.allclose(aux["w_new"], np.array(Wl), rtol=1e-12, atol=1e-14)
        Wl = W.astype(np.float64).tolist()      # follow the oracle's fp32 storage of W


def test_scalar_loops_full_momentum_4x4():
    g = rng(20)
    hp = O.HParams(beta1=0.5, beta2=0.5, clip=1.0)
    blk = O.Block(4, 4, mom_mode=O.MOM_FULL, weight_decay=0.25)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    W = g.standard_normal((4, 4)).astype(np.float32)
    ml, vl = LO.zeros(4, 4), LO.zeros(4, 4)
    for t in range(1, 4):
        G = g.standard_normal((4, 4)).astype(np.float32)
        Wl, ml, vl = LO.full_step(W.astype(np.float64).tolist(), G.astype(np.float64).tolist(), ml, vl,
                                  0.5, 0.5, 1e-8, 1.0, 0.25, 0.125)
        W, st, aux = O.step_block(blk, hp, W, G, st, t, 0.125, state_dtype=np.float64, want_aux=True)
        assert np.allclose(aux["w_new"], np.array(Wl), rtol=1e-13, atol=1e-15)
        assert np.allclose(st["m"], np.array(ml), rtol=1e-14)


# ---------------------------------------------------------------------------
# P10: blockwise second moment
# ---------------------------------------------------------------------------
def test_P10_blockwise_v_reductions():
    g = rng(13)
    m_, n_ = 12, 5
    hp = O.HParams()
    Gs = [g.standard_normal((m_, n_)).astype(np.float32) for _ in range(4)]
    W0 = g.standard_normal((m_, n_)).astype(np.float32)

    def run(blk, Gl):
        st = O.init_state([blk], hp, dtype=np.float64)[0]
        W = W0.copy()
        for t, G in enumerate(Gl, 1):
            W, st, aux = O.step_block(blk, hp, W, G, st, t, 1e-2, state_dtype=np.float64, want_aux=True)
        return W, st, aux

    # (a) per-element run, then average v over groups == group run's v (EMA and mean commute)
    We, se, _ = run(O.Block(m_, n_, v_mode=O.V_ELEMENT), Gs)
    for gr in (1, 3, 12):
        Wg, sg, aux = run(O.Block(m_, n_, v_mode=O.V_ROWGROUP, v_group_rows=gr), Gs)
        want = se["v"].reshape(m_ // gr, gr * n_).mean(axis=1)
        assert np.allclose(sg["v"], want, rtol=1e-13)
        assert aux["v_full"].shape == (m_, n_)
        for i in range(m_):
            assert np.all(aux["v_full"][i] == sg["v"][i // gr])
    Ww, sw, _ = run(O.Block(m_, n_, v_mode=O.V_WHOLE), Gs)
    assert sw["v"].shape == (1,) and sw["v"][0] == pytest.approx(se["v"].mean(), rel=1e-13)
    # (b) one column, group of one row == per element
    Gc = [x[:, :1].copy() for x in Gs]
    W0c = W0[:, :1].copy()
    st1 = O.init_state([O.Block(m_, 1)], hp, dtype=np.float64)[0]
    st2 = O.init_state([O.Block(m_, 1, v_mode=O.V_ROWGROUP, v_group_rows=1)], hp, dtype=np.float64)[0]
    Wa, Wb = W0c.copy(), W0c.copy()
    for t, G in enumerate(Gc, 1):
        Wa, st1, _ = O.step_block(O.Block(m_, 1), hp, Wa, G, st1, t, 1e-2, state_dtype=np.float64)
        Wb, st2, _ = O.step_block(O.Block(m_, 1, v_mode=O.V_ROWGROUP, v_group_rows=1), hp, Wb, G, st2, t, 1e-2,
                                  state_dtype=np.float64)
    assert np.array_equal(Wa, Wb) and np.array_equal(st1["v"], st2["v"])
    # (c) constant-magnitude gradient: whole-block v == per-element v
    Gk = [(np.sign(x) * 0.5).astype(np.float32) for x in Gs]
    Wk1, _, _ = run(O.Block(m_, n_, v_mode=O.V_ELEMENT), Gk)
    Wk2, _, _ = run(O.Block(m_, n_, v_mode=O.V_WHOLE), Gk)
    assert np.array_equal(Wk1, Wk2)


def test_no_momentum_block_uses_raw_gradient_and_lr_scale():
    g = rng(14)
    hp = O.HParams()
    blk = O.Block(6, 3, mom_mode=O.MOM_NONE, lr_scale=0.75, weight_decay=0.1)
    st = O.init_state([blk], hp)[0]
    assert set(st) == {"v"}
    W0 = g.standard_normal((6, 3)).astype(np.float32)
    G = g.standard_normal((6, 3)).astype(np.float32)
    _, st, aux = O.step_block(blk, hp, W0, G, st, 1, 1e-2, want_aux=True)
    G64, W64 = G.astype(np.float64), W0.astype(np.float64)
    u = np.clip(G64 / (np.sqrt(0.05 * G64 ** 2) + 1e-8), -1, 1)
    assert np.allclose(aux["w_new"], W64 - 0.75e-2 * (u + 0.1 * W64), atol=1e-15)


def test_ablation_without_bias_correction_uses_the_product():
    m_, n_, r = 10, 8, 2
    hp = O.HParams(bias_correction=0, seed=4)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    G = lowrank_grads(m_, n_, 4, 1, seed=15)[0]
    _, st, aux = O.step_block(blk, hp, np.zeros((m_, n_), np.float32), G, st, 1, 1e-2,
                              state_dtype=np.float64, want_aux=True)
    assert np.allclose(aux["mc"], st["L"] @ st["R"], atol=1e-15)


# ---------------------------------------------------------------------------
# P12: the T > 1 reading (normal equations; the paper itself does not pin it)
# ---------------------------------------------------------------------------
def test_P12_projection_step_is_least_squares_with_R_held():
    m_, n_, r, T = 20, 16, 3, 4
    b1 = 0.9
    hp = O.HParams(T=T, seed=21)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    Gs = lowrank_grads(m_, n_, 6, 9, seed=16)
    st = O.init_state([blk], hp, dtype=np.float64)[0]
    W = np.zeros((m_, n_), np.float32)
    for t in range(1, 10):
        prev = st
        W, st, aux = O.step_block(blk, hp, W, Gs[t - 1], st, t, 1e-3, state_dtype=np.float64, want_aux=True)
        Q = st["R"]
        assert np.allclose(Q @ Q.T, np.eye(r), atol=1e-12)            # re-gauged rows stay orthonormal
        if (t - 1) % T == 0:
            # refresh step: Alg. 2 then a re-gauge that keeps the product
            Lg, Rg = O.refresh_gd(aux["M"], prev["L"], prev["R"], hp.K)
            assert np.allclose(st["L"] @ st["R"], Lg @ Rg, atol=1e-13)
        else:
            assert np.array_equal(st["R"], prev["R"])
            Lls = np.linalg.lstsq(Q.T, aux["M"].T, rcond=None)[0].T      # library least squares
            assert np.allclose(st["L"], Lls, atol=1e-12)
            assert np.abs(aux["r"] @ Q.T).max() < 1e-13                  # residual orthogonal to the rows
            G = Gs[t - 1].astype(np.float64)
            assert np.allclose(st["L"], b1 * prev["L"] + (1 - b1) * G @ Q.T, atol=1e-13)
            assert np.allclose(aux["mc"], G + b1 * (prev["L"] - G @ Q.T) @ Q, atol=1e-13)


def test_regauge_keeps_product_and_orthonormalises():
    g = rng(17)
    L, R = g.standard_normal((9, 3)), g.standard_normal((3, 11))
    L2, R2 = O.regauge(L, R)
    assert np.allclose(L2 @ R2, L @ R, atol=1e-13)
    assert np.allclose(R2 @ R2.T, np.eye(3), atol=1e-13)


def test_projection_product_is_gauge_independent():
    g = rng(18)
    M = g.standard_normal((7, 9))
    R = g.standard_normal((2, 9))
    C = g.standard_normal((2, 2)) + 3 * np.eye(2)
    assert np.allclose(O.lstsq_L(M, R) @ R, O.lstsq_L(M, C @ R) @ (C @ R), atol=1e-12)


# ---------------------------------------------------------------------------
# stability of the literal solver on the synthetic gradient model (finite state)
# ---------------------------------------------------------------------------
def test_literal_solver_stays_finite_and_tracks_on_synthetic_gradients():
    m_, n_, r, T = 96, 64, 8, 40
    hp = O.HParams(seed=2)
    blk = O.Block(m_, n_, mom_mode=O.MOM_LOWRANK, rank=r)
    Gs = lowrank_grads(m_, n_, 32, T, seed=19)
    st = O.init_state([blk], hp)[0]
    W = np.zeros((m_, n_), np.float32)
    ratios = []
    for t in range(1, T + 1):
        W, st, aux = O.step_block(blk, hp, W, Gs[t - 1], st, t, 1e-3, want_aux=True)
        assert np.isfinite(st["L"]).all() and np.isfinite(st["R"]).all() and np.isfinite(W).all()
        ratios.append(np.linalg.norm(aux["r"]) / np.linalg.norm(aux["M"]))
    assert ratios[0] > 0.9 and ratios[-1] < 0.3


# ---------------------------------------------------------------------------------------------------
# Pre-step of the paper's runs (Sec. 5.1, set-ups): global gradient-norm clipping, warm-up + cosine LR
# ---------------------------------------------------------------------------------------------------
def test_global_grad_scale_closed_form_and_brute_force():
    blocks = [O.Block(2, 2, grad_dtype=O.F32), O.Block(1, 1, grad_dtype=O.F32), O.Block(2, 1, grad_dtype=O.BF16)]
    Gs = [np.array([[3.0, 0.0], [0.0, 0.0]], np.float32), np.array([[4.0]], np.float32),
          O.f64_to_bf16_bits(np.array([[12.0], [0.0]]))]
    scale, norm = O.global_grad_scale(blocks, Gs, 1.0)
    assert norm == 13.0                                    # 3-4-12: sqrt(9 + 16 + 144)
    assert scale == 1.0 / (13.0 + 1e-6)
    assert O.global_grad_scale(blocks, Gs, 20.0)[0] == 1.0  # below the threshold: untouched
    rng = np.random.default_rng(0)
    blocks = [O.Block(5, 3, grad_dtype=O.F32), O.Block(7, 1, grad_dtype=O.F32)]
    Gs = [rng.standard_normal((5, 3)).astype(np.float32), rng.standard_normal((7, 1)).astype(np.float32)]
    tot = 0.0
    for g in Gs:                                            # scalar loop
        for x in g.reshape(-1):
            tot += float(x) * float(x)
    scale, norm = O.global_grad_scale(blocks, Gs, 0.5)
    assert abs(norm - math.sqrt(tot)) < 1e-12 and abs(scale - 0.5 / (math.sqrt(tot) + 1e-6)) < 1e-15
    assert scale * norm <= 0.5                              # the clipped gradient is inside the ball


def test_step_with_global_clipping_sees_the_scaled_gradient():
    """Clipping is linear pre-processing: a step with clipping on G equals a step without clipping on the
    explicitly scaled gradient; a threshold above the norm changes nothing."""
    rng = np.random.default_rng(4)
    blocks = [O.Block(12, 10, mom_mode=O.MOM_LOWRANK, rank=3, weight_decay=0.1),
              O.Block(6, 4, mom_mode=O.MOM_FULL, v_mode=O.V_ROWGROUP, v_group_rows=2),
              O.Block(5, 1, mom_mode=O.MOM_NONE, lr_scale=0.75)]
    hp = O.HParams(K=3, T=1)
    Ws = [rng.standard_normal((b.rows, b.cols)).astype(np.float32) for b in blocks]
    Gs = [rng.standard_normal((b.rows, b.cols)).astype(np.float32) for b in blocks]
    st = O.init_state(blocks, hp)
    scale, norm = O.global_grad_scale(blocks, Gs, 1.0)
    assert norm > 1.0 and scale < 1.0
    W1, S1 = O.step(blocks, hp, Ws, Gs, st, 1, 1e-2, grad_clip=1.0)
    W2, S2 = Ws, st
    W2 = list(W2); S2 = list(S2)
    for i, b in enumerate(blocks):
        W2[i], S2[i], _ = O.step_block(b, hp, Ws[i], Gs[i], st[i], 1, 1e-2, g_scale=scale)
    for a, b_ in zip(W1, W2):
        np.testing.assert_array_equal(a, b_)
    # scaled fp32 copies of G give the same result up to the rounding of the copy
    G3 = [(g.astype(np.float64) * scale).astype(np.float32) for g in Gs]
    W3, _ = O.step(blocks, hp, Ws, G3, st, 1, 1e-2)
    for a, b_ in zip(W1, W3):
        np.testing.assert_allclose(a, b_, rtol=0, atol=2e-7)
    W4, S4 = O.step(blocks, hp, Ws, Gs, st, 1, 1e-2, grad_clip=10.0 * norm)
    W5, S5 = O.step(blocks, hp, Ws, Gs, st, 1, 1e-2)
    for a, b_ in zip(W4, W5):
        np.testing.assert_array_equal(a, b_)


def test_lr_schedule_warmup_then_cosine():
    peak, lo, wu, tot = 6e-4, 6e-5, 2000, 100000
    f = lambda t: O.lr_cosine_warmup(t, peak, lo, wu, tot)
    assert f(1) == peak / wu and f(1000) == peak / 2 and f(wu) == peak          # linear warm-up reaching the peak
    assert f(tot) == lo and f(tot + 5) == lo                                     # floor from the last step on
    mid = (wu + tot) // 2
    assert abs(f(mid) - 0.5 * (peak + lo)) < 1e-12                               # half-way down at the mid-point
    xs = [f(t) for t in range(wu, tot + 1, 997)]
    assert all(a >= b for a, b in zip(xs, xs[1:]))                               # monotone decay
    q = wu + (tot - wu) // 4
    assert abs(f(q) - (lo + 0.5 * (peak - lo) * (1 + math.cos(math.pi / 4)))) < 1e-12


# ---------------------------------------------------------------------------------------------------
# Scale-normalised Alg. 2 (an option beyond the paper)
# ---------------------------------------------------------------------------------------------------
def test_normalised_alg2_is_scale_invariant_and_literal_alg2_is_not():
    rng = np.random.default_rng(11)
    m_, n_, r = 14, 11, 3
    M = rng.standard_normal((m_, r)) @ rng.standard_normal((r, n_)) + 0.05 * rng.standard_normal((m_, n_))
    L0 = 0.3 * rng.standard_normal((m_, r))
    R0 = 0.3 * rng.standard_normal((r, n_))
    L1, R1 = O.refresh_gd(M, L0, R0, 5, normalise=True)
    for c in (1e-4, 37.0, 1e4):
        Lc, Rc = O.refresh_gd(c * M, math.sqrt(c) * L0, math.sqrt(c) * R0, 5, normalise=True)
        np.testing.assert_allclose(Lc, math.sqrt(c) * L1, rtol=1e-10, atol=0)
        np.testing.assert_allclose(Rc, math.sqrt(c) * R1, rtol=1e-10, atol=0)
    # the printed iteration does not have this property: at c = 37 it blows up, at c = 1e-4 it barely moves
    La, Ra = O.refresh_gd(M, L0, R0, 5)
    with np.errstate(over="ignore", invalid="ignore"):
        Lb, Rb = O.refresh_gd(37.0 * M, math.sqrt(37.0) * L0, math.sqrt(37.0) * R0, 5)
    assert not np.allclose(Lb @ Rb, 37.0 * (La @ Ra), rtol=1e-3)
    Ls, Rs = O.refresh_gd(1e-4 * M, 1e-2 * L0, 1e-2 * R0, 5)
    moved_literal = np.linalg.norm(Ls - 1e-2 * L0) / np.linalg.norm(1e-2 * L0)
    moved_normalised = np.linalg.norm(L1 - L0) / np.linalg.norm(L0)
    assert moved_literal < 0.02 * moved_normalised


def test_normalised_alg2_descends_at_any_scale_and_reduces_to_the_literal_one():
    rng = np.random.default_rng(12)
    m_, n_, r = 20, 16, 4
    M = rng.standard_normal((m_, r)) @ rng.standard_normal((r, n_))
    for c in (1e-3, 1.0, 1e3):
        L, R = np.zeros((m_, r)), math.sqrt(c) * rng.standard_normal((r, n_)) / math.sqrt(n_)
        errs = [np.linalg.norm(L @ R - c * M)]
        for _ in range(12):
            L, R = O.refresh_gd(c * M, L, R, 5, normalise=True)
            errs.append(np.linalg.norm(L @ R - c * M))
        assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:]))          # monotone
        assert errs[-1] < 0.2 * errs[0]                                            # and it gets somewhere
    # normaliser 1: rank 1, unit row, L = 0  =>  the first iteration is the printed one
    R0 = np.zeros((1, n_)); R0[0, 3] = 1.0
    La, Ra = O.refresh_gd(M, np.zeros((m_, 1)), R0, 2)
    Lb, Rb = O.refresh_gd(M, np.zeros((m_, 1)), R0, 2, normalise=True)
    np.testing.assert_array_equal(La, Lb)
    np.testing.assert_array_equal(Ra, Rb)


def test_regauge_of_rank_deficient_factors_is_an_error_in_the_oracle():
    """The product-preserving re-expression (reading of T > 1) needs R R^T positive definite.  The oracle does not
    paper over a rank-deficient R: the library routine raises, e.g. for the literal zero start of Alg. 1."""
    L, R = np.zeros((6, 2)), np.zeros((2, 5))
    with pytest.raises(np.linalg.LinAlgError):
        O.regauge(L, R)
    blk = O.Block(6, 5, mom_mode=O.MOM_LOWRANK, rank=2)
    hp = O.HParams(T=2, seed=0)
    st = O.init_state([blk], hp)[0]
    G = np.arange(30, dtype=np.float32).reshape(6, 5) / 30
    with pytest.raises(np.linalg.LinAlgError):
        O.step_block(blk, hp, np.zeros((6, 5), np.float32), G, st, 1, 1e-3)
    # with Alg. 2 every step (T = 1) the same start is well defined: the factors stay zero and m^c = G
    hp1 = O.HParams(T=1, seed=0)
    _, new, aux = O.step_block(blk, hp1, np.zeros((6, 5), np.float32), G, st, 1, 1e-3, want_aux=True)
    assert not new["L"].any() and not new["R"].any()
    assert np.allclose(aux["mc"], G.astype(np.float64), rtol=1e-14, atol=0.0)
