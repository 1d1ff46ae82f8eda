"""Brute-force form of the neighbor-mode block backward: every output element as an explicit index sum.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Pure Python floats and nested loops, no numpy, no
matrix routine: it exists to pin the numpy oracle on tiny inputs (a transposed operand, a wrong index
or a dropped term in either one shows up as a disagreement) and as the slowest leg of the benchmark's
CPU baseline.  It imports nothing from the numpy oracle or from the HIP path.

What it computes (Alg. 3, neighbor branch; Sec. 3.2 skip; Sec. 3.3 recompute; Sec. 3.4 Eq. (2)),
tokens i, model columns j, l, hidden columns k, rank index q:
    rstd_i = (1/d sum_j H_ij^2 + eps)^(-1/2),  N_ij = H_ij rstd_i,  U_ij = N_ij gamma_j
    G_ik = sum_j U_ij Wg_kj,  Z_ik = sum_j U_ij Wu_kj,  s = 1/(1+exp(-G)),  A = G s Z
    dA_ik = sum_j dOut_ij Wd_jk
    dZ_ik = dA_ik G_ik s_ik,  dG_ik = dA_ik Z_ik (s_ik + G_ik s_ik (1 - s_ik))
    dU_ij = sum_k (dG_ik Wg_kj + dZ_ik Wu_kj)
    dgamma_j = sum_i dU_ij N_ij
    dX_ij = dOut_ij + rstd_i (dU_ij gamma_j - N_ij (1/d) sum_l dU_il gamma_l N_il)
    dWg_kj = sum_q [sum_i dG_ik (sum_l U_il Pg_lq)] Pg_jq      (Eq. (2): G_y (x^T V1) V1^T)
    dWu_kj = sum_q [sum_i dZ_ik (sum_l U_il Pu_lq)] Pu_jq
    dWd_jk = sum_q [sum_i dOut_ij (sum_l A_il Pd_lq)] Pd_kq
"""
from __future__ import annotations

import math


def _lists(x):
    return [[float(v) for v in row] for row in x]


def block_bwd_skip_loops(H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, eps=1e-6):
    """All arguments are nested sequences (rows of numbers); returns nested lists."""
    H, dOut, Wg, Wu, Wd = _lists(H), _lists(dOut), _lists(Wg), _lists(Wu), _lists(Wd)
    Pg, Pu, Pd = _lists(Pg), _lists(Pu), _lists(Pd)
    gamma = [float(v) for v in gamma]
    b, d, f = len(H), len(H[0]), len(Wg)
    rg, ru, rd = len(Pg[0]), len(Pu[0]), len(Pd[0])

    rstd = [0.0] * b
    N = [[0.0] * d for _ in range(b)]
    U = [[0.0] * d for _ in range(b)]
    for i in range(b):
        ss = 0.0
        for j in range(d):
            ss += H[i][j] * H[i][j]
        rstd[i] = 1.0 / math.sqrt(ss / d + eps)
        for j in range(d):
            N[i][j] = H[i][j] * rstd[i]
            U[i][j] = N[i][j] * gamma[j]

    A = [[0.0] * f for _ in range(b)]
    dG = [[0.0] * f for _ in range(b)]
    dZ = [[0.0] * f for _ in range(b)]
    for i in range(b):
        for k in range(f):
            g = z = da = 0.0
            for j in range(d):
                g += U[i][j] * Wg[k][j]
                z += U[i][j] * Wu[k][j]
                da += dOut[i][j] * Wd[j][k]
            s = 1.0 / (1.0 + math.exp(-g))
            A[i][k] = g * s * z
            dZ[i][k] = da * g * s
            dG[i][k] = da * z * (s + g * s * (1.0 - s))

    dU = [[0.0] * d for _ in range(b)]
    for i in range(b):
        for j in range(d):
            acc = 0.0
            for k in range(f):
                acc += dG[i][k] * Wg[k][j] + dZ[i][k] * Wu[k][j]
            dU[i][j] = acc

    dgamma = [0.0] * d
    dX = [[0.0] * d for _ in range(b)]
    for i in range(b):
        dot = 0.0
        for l in range(d):
            dot += dU[i][l] * gamma[l] * N[i][l]
        dot /= d
        for j in range(d):
            dgamma[j] += dU[i][j] * N[i][j]
            dX[i][j] = dOut[i][j] + rstd[i] * (dU[i][j] * gamma[j] - N[i][j] * dot)

    def eq2(Gy, X, P, m, n, r):
        """[m x n] = sum_q (sum_i Gy_i,row (sum_l X_il P_lq)) P_col,q with Gy [b x m], X [b x n], P [n x r]."""
        T = [[0.0] * r for _ in range(b)]
        for i in range(b):
            for q in range(r):
                acc = 0.0
                for l in range(n):
                    acc += X[i][l] * P[l][q]
                T[i][q] = acc
        C = [[0.0] * r for _ in range(m)]
        for row in range(m):
            for q in range(r):
                acc = 0.0
                for i in range(b):
                    acc += Gy[i][row] * T[i][q]
                C[row][q] = acc
        W = [[0.0] * n for _ in range(m)]
        for row in range(m):
            for col in range(n):
                acc = 0.0
                for q in range(r):
                    acc += C[row][q] * P[col][q]
                W[row][col] = acc
        return W

    return dict(dX=dX, dgamma=dgamma, dWg=eq2(dG, U, Pg, f, d, rg), dWu=eq2(dZ, U, Pu, f, d, ru),
                dWd=eq2(dOut, A, Pd, d, f, rd))
