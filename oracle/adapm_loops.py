"""Scalar-loop brute force of Alg. 1 + Alg. 2 for tiny blocks.

TEST INFRASTRUCTURE ONLY.  No numpy, no matrix products: every sum of Alg. 1
(momentum m_t, residual r_t of eq. 3, correction of eq. 4, update) and Alg. 2
(the two printed gradients, simultaneous update) is written as nested loops over
python floats, so the vectorised oracle can be checked against it on 4 x 4
blocks.  Per-element second moment, T = 1, fp64 throughout, no storage rounding.
"""
import math


def zeros(a, b):
    return [[0.0] * b for _ in range(a)]


def lowrank_step(W, G, L, R, v, beta1, beta2, eps, clip, lam, lr, K):
    """One step of Alg. 1 on an m x n block given as lists of lists.
    Returns (W_new, L_new, R_new, v_new, mc, res)."""
    m, n, r = len(W), len(W[0]), len(R)
    # m_t = (1 - beta1) G + beta1 L R
    M = zeros(m, n)
    for i in range(m):
        for j in range(n):
            a = 0.0
            for k in range(r):
                a += L[i][k] * R[k][j]
            M[i][j] = (1.0 - beta1) * G[i][j] + beta1 * a
    # Alg. 2
    Lc = [row[:] for row in L]
    Rc = [row[:] for row in R]
    for it in range(1, K + 1):
        eta = 0.5 * (1.0 + math.cos(math.pi * it / K))
        E = zeros(m, n)
        for i in range(m):
            for j in range(n):
                a = 0.0
                for k in range(r):
                    a += Lc[i][k] * Rc[k][j]
                E[i][j] = a - M[i][j]
        dL = zeros(m, r)
        for i in range(m):
            for k in range(r):
                a = 0.0
                for j in range(n):
                    a += E[i][j] * Rc[k][j]
                dL[i][k] = a
        dR = zeros(r, n)
        for k in range(r):
            for j in range(n):
                a = 0.0
                for i in range(m):
                    a += Lc[i][k] * E[i][j]
                dR[k][j] = a
        for i in range(m):
            for k in range(r):
                Lc[i][k] -= eta * dL[i][k]
        for k in range(r):
            for j in range(n):
                Rc[k][j] -= eta * dR[k][j]
    # residual, correction, second moment, update
    Wn, vn, mc, res = zeros(m, n), zeros(m, n), zeros(m, n), zeros(m, n)
    for i in range(m):
        for j in range(n):
            b = 0.0
            for k in range(r):
                b += Lc[i][k] * Rc[k][j]
            res[i][j] = b - M[i][j]
            mc[i][j] = M[i][j] - beta1 * res[i][j] / (1.0 - beta1)
            vn[i][j] = beta2 * v[i][j] + (1.0 - beta2) * G[i][j] * G[i][j]
            u = mc[i][j] / (math.sqrt(vn[i][j]) + eps)
            u = max(-clip, min(clip, u))
            Wn[i][j] = W[i][j] - lr * (u + lam * W[i][j])
    return Wn, Lc, Rc, vn, mc, res


def full_step(W, G, mom, v, beta1, beta2, eps, clip, lam, lr):
    """Full-momentum block (eq. 5) with the same update line."""
    m, n = len(W), len(W[0])
    Wn, mn, vn = zeros(m, n), zeros(m, n), zeros(m, n)
    for i in range(m):
        for j in range(n):
            mn[i][j] = (1.0 - beta1) * G[i][j] + beta1 * mom[i][j]
            vn[i][j] = beta2 * v[i][j] + (1.0 - beta2) * G[i][j] * G[i][j]
            u = mn[i][j] / (math.sqrt(vn[i][j]) + eps)
            u = max(-clip, min(clip, u))
            Wn[i][j] = W[i][j] - lr * (u + lam * W[i][j])
    return Wn, mn, vn
