"""CPU oracle for MeCeFO's neighbor-mode (degraded) transformer-block backward.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, numpy
implementation (fp64 unless a dtype is passed) written from the paper:
  * Sec. 3.2 / Fig. 2 / Alg. 3 "skip the MHA connection": in the backward pass the
    attention branch is dropped, the activation gradient goes through the residual.
  * Sec. 3.3 / Alg. 2-3: only the input of the FFN module is kept; every other FFN
    activation is recomputed in the backward pass.
  * Sec. 3.4 Eq. (2): G_W = G_y x^T  ~=  G_y (x^T V1) V1^T with V1 the top-r right
    singular vectors of W (y = W x, W in R^{m x n}).
  * Sec. 2 "Transformer models": LLaMA block = MHA + FFN(W_gate, W_up, W_down), each
    with normalisation and a residual connection.
It shares no code with the HIP path and imports nothing from it.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may call it.

Every function below is pinned by tests that do not re-type its formula: finite
differences, torch.autograd of an independently written module, the full-rank
identity, projector algebra, invariants, and a brute-force index-sum form in pure Python
(oracle/mecefo_loops.py) on tiny inputs (see tests/test_oracle_pins.py).
The paper prints no per-layer numeric example, so no printed value pins it.

Row-major conventions (tokens along rows):
  b tokens, d = d_model, f = d_ff, r = rank.
  H [b,d] stored FFN-module input (residual stream after attention, before the norm)
  U = RMSNorm(H) * gamma;  Wg, Wu [f,d];  Wd [d,f];  G = U Wg^T, Z = U Wu^T;
  S = silu(G);  A = S * Z;  Y = A Wd^T;  Out = H + Y.
Readings of points the paper leaves open (listed in the design notes): SwiGLU FFN
without biases; pre-norm RMSNorm with gain; the stored tensor is H; the FFN-norm
gain gets its exact gradient, the attention-norm gain gets none.
"""
from __future__ import annotations

import numpy as np

SIDE_INPUT = 0   # Eq. (2) as printed: project the layer input x (P in R^{n_in x r})
SIDE_OUTPUT = 1  # project the output gradient instead (P in R^{m_out x r})


def _f(x, dtype):
    return np.asarray(x, dtype=dtype)


# --------------------------------------------------------------------------- norm
def rmsnorm_fwd(H, gamma, eps, dtype=np.float64):
    """rstd_i = (mean_j H_ij^2 + eps)^(-1/2);  N = H * rstd;  U = N * gamma."""
    H = _f(H, dtype)
    rstd = 1.0 / np.sqrt(np.mean(H * H, axis=1, keepdims=True) + eps)
    N = H * rstd
    U = N * _f(gamma, dtype)[None, :]
    return U, N, rstd


def rmsnorm_bwd(dU, N, rstd, gamma, dtype=np.float64):
    """Gradient of U = N*gamma, N = H*rstd(H) with respect to H and gamma."""
    dU = _f(dU, dtype)
    dN = dU * _f(gamma, dtype)[None, :]
    dgamma = np.sum(dU * N, axis=0)
    dH = rstd * (dN - N * np.mean(dN * N, axis=1, keepdims=True))
    return dH, dgamma


# --------------------------------------------------------------------------- FFN
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def ffn_fwd_recompute(U, Wg, Wu, Wd=None, dtype=np.float64):
    """Sec. 3.3 Rcomp: rebuild the FFN activations from the module input U.

    Returns G, Z, A (and Y = A Wd^T when Wd is given; the backward never needs Y).
    """
    U, Wg, Wu = _f(U, dtype), _f(Wg, dtype), _f(Wu, dtype)
    G = U @ Wg.T
    Z = U @ Wu.T
    A = (G * sigmoid(G)) * Z
    Y = None if Wd is None else A @ _f(Wd, dtype).T
    return G, Z, A, Y


def ffn_dgrad(dY, G, Z, Wg, Wu, Wd, dtype=np.float64):
    """Exact activation gradients through the FFN (Dgrad is never approximated, Sec. 3.3-3.4)."""
    dY, Wg, Wu, Wd = _f(dY, dtype), _f(Wg, dtype), _f(Wu, dtype), _f(Wd, dtype)
    sg = sigmoid(G)
    S = G * sg
    dA = dY @ Wd
    dZ = dA * S
    dG = dA * Z * (sg * (1.0 + G * (1.0 - sg)))
    dU = dG @ Wg + dZ @ Wu
    return dU, dG, dZ


def wgrad_exact(Gy, X, dtype=np.float64):
    """G_W = G_y x^T summed over tokens: [b,m]^T [b,n] -> [m,n] (Sec. 3.4, left side of Eq. 2)."""
    return _f(Gy, dtype).T @ _f(X, dtype)


def wgrad_lowrank(Gy, X, P, side=SIDE_INPUT, dtype=np.float64):
    """Eq. (2) in its printed bracket order: G_y (x^T V1) V1^T.

    Gy [b,m] output gradient, X [b,n] layer input, result [m,n].
    SIDE_INPUT : P [n,r];  T = X P  [b,r];  C = Gy^T T  [m,r];  G_W = C P^T.
    SIDE_OUTPUT: P [m,r];  T = Gy P [b,r];  C = X^T T   [n,r];  G_W = (C P^T)^T = P C^T.
    """
    Gy, X, P = _f(Gy, dtype), _f(X, dtype), _f(P, dtype)
    if side == SIDE_INPUT:
        T = X @ P
        C = Gy.T @ T
        return C @ P.T
    T = Gy @ P
    C = X.T @ T
    return (C @ P.T).T


def projection_from_svd(W, r, side=SIDE_INPUT):
    """V1 = V[:, :r] of W = U Sigma V^T (Sec. 3.4); for SIDE_OUTPUT the top-r left vectors."""
    W = np.asarray(W, dtype=np.float64)
    Uw, _, Vh = np.linalg.svd(W, full_matrices=False)
    if r > min(W.shape):
        raise ValueError("rank exceeds min(m, n)")
    return Vh[:r].T.copy() if side == SIDE_INPUT else Uw[:, :r].copy()


def ffn_bwd_exact(U, dY, Wg, Wu, Wd, dtype=np.float64):
    """Recompute + exact Dgrad + exact Wgrad of the FFN (the un-approximated reference)."""
    G, Z, A, _ = ffn_fwd_recompute(U, Wg, Wu, dtype=dtype)
    dU, dG, dZ = ffn_dgrad(dY, G, Z, Wg, Wu, Wd, dtype=dtype)
    return dict(dU=dU, dWg=wgrad_exact(dG, U, dtype), dWu=wgrad_exact(dZ, U, dtype),
                dWd=wgrad_exact(dY, A, dtype))


def ffn_bwd_lowrank(U, dY, Wg, Wu, Wd, Pg, Pu, Pd, side=SIDE_INPUT, dtype=np.float64):
    """Alg. 3, neighbor branch, FFN part: recompute, exact Dgrad, Eq. (2) for gate/up/down."""
    G, Z, A, _ = ffn_fwd_recompute(U, Wg, Wu, dtype=dtype)
    dU, dG, dZ = ffn_dgrad(dY, G, Z, Wg, Wu, Wd, dtype=dtype)
    Uc = _f(U, dtype)
    return dict(dU=dU,
                dWg=wgrad_lowrank(dG, Uc, Pg, side, dtype),
                dWu=wgrad_lowrank(dZ, Uc, Pu, side, dtype),
                dWd=wgrad_lowrank(dY, A, Pd, side, dtype))


def block_bwd_skip(H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, eps=1e-6, side=SIDE_INPUT,
                   dtype=np.float64):
    """Neighbor-mode backward of one block (Alg. 3: recompute, Eq. (2), skip MHA).

    Out = H + FFN(RMSNorm(H)); the block input X reaches H through the residual
    (H = X + MHA(..)), and the MHA branch is cut in the backward pass, hence
    dX = dH.  No MHA parameter receives a gradient.  gamma=None means no norm (U = H).
    """
    H, dOut = _f(H, dtype), _f(dOut, dtype)
    if gamma is None:
        U = H
    else:
        U, N, rstd = rmsnorm_fwd(H, gamma, eps, dtype)
    g = ffn_bwd_lowrank(U, dOut, Wg, Wu, Wd, Pg, Pu, Pd, side, dtype)
    if gamma is None:
        dHn, dgamma = g["dU"], None
    else:
        dHn, dgamma = rmsnorm_bwd(g["dU"], N, rstd, gamma, dtype)
    dH = dOut + dHn
    return dict(dX=dH, dgamma=dgamma, dWg=g["dWg"], dWu=g["dWu"], dWd=g["dWd"])


def block_bwd_skip_exact_wgrad(H, dOut, gamma, Wg, Wu, Wd, eps=1e-6, dtype=np.float64):
    """Same skip + recompute, but with exact FFN weight gradients (no Eq. (2))."""
    H, dOut = _f(H, dtype), _f(dOut, dtype)
    U, N, rstd = rmsnorm_fwd(H, gamma, eps, dtype)
    g = ffn_bwd_exact(U, dOut, Wg, Wu, Wd, dtype)
    dHn, dgamma = rmsnorm_bwd(g["dU"], N, rstd, gamma, dtype)
    return dict(dX=dOut + dHn, dgamma=dgamma, dWg=g["dWg"], dWu=g["dWu"], dWd=g["dWd"])


# ------------------------------------------------------ full block (standard mode)
def _rope_tables(seq, dh, theta=10000.0):
    inv = theta ** (-np.arange(0, dh, 2, dtype=np.float64) / dh)
    ang = np.arange(seq, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)          # [seq, dh/2]


def _rope(x, cos, sin, inverse=False):
    """Rotate pairs (x[..., :dh/2], x[..., dh/2:]) by the position angle; x [B,h,S,dh]."""
    h2 = x.shape[-1] // 2
    x1, x2 = x[..., :h2], x[..., h2:]
    s = -sin if inverse else sin
    return np.concatenate([x1 * cos - x2 * s, x1 * s + x2 * cos], axis=-1)


def mha_fwd(X, g_attn, Wq, Wk, Wv, Wo, heads, batch, seq, eps=1e-6, dtype=np.float64):
    """Pre-norm causal multi-head attention with RoPE; returns branch output and a cache."""
    X = _f(X, dtype)
    d = X.shape[1]
    dh = d // heads
    Xn, N, rstd = rmsnorm_fwd(X, g_attn, eps, dtype)

    def split(t):
        return t.reshape(batch, seq, heads, dh).transpose(0, 2, 1, 3)

    cos, sin = (_f(t, dtype) for t in _rope_tables(seq, dh))
    Q = _rope(split(Xn @ _f(Wq, dtype).T), cos, sin)
    K = _rope(split(Xn @ _f(Wk, dtype).T), cos, sin)
    V = split(Xn @ _f(Wv, dtype).T)
    sc = (Q @ K.transpose(0, 1, 3, 2)) / dtype(np.sqrt(dh))
    mask = np.triu(np.ones((seq, seq), dtype=bool), 1)
    sc = np.where(mask, -np.inf, sc)
    mx = sc.max(axis=-1, keepdims=True)
    sc = sc - mx
    Pm = np.exp(sc)
    den = Pm.sum(axis=-1, keepdims=True)
    Pm /= den
    L = (mx + np.log(den))[..., 0]          # log-sum-exp of the scaled, masked scores [B,h,S]
    O = (Pm @ V).transpose(0, 2, 1, 3).reshape(batch * seq, d)
    M = O @ _f(Wo, dtype).T
    cache = dict(Xn=Xn, N=N, rstd=rstd, Q=Q, K=K, V=V, Pm=Pm, O=O, L=L, cos=cos, sin=sin,
                 heads=heads, batch=batch, seq=seq)
    return M, cache


def mha_bwd(dM, cache, g_attn, Wq, Wk, Wv, Wo):
    """Backward of mha_fwd: gradient to the block input through the attention branch,
    and the gradients of Wq, Wk, Wv, Wo and the attention-norm gain."""
    c = cache
    heads, batch, seq = c["heads"], c["batch"], c["seq"]
    d = dM.shape[1]
    dh = d // heads
    Wq, Wk, Wv, Wo = (_f(w, np.float64) for w in (Wq, Wk, Wv, Wo))
    dWo = dM.T @ c["O"]
    dO = (dM @ Wo).reshape(batch, seq, heads, dh).transpose(0, 2, 1, 3)
    dPm = dO @ c["V"].transpose(0, 1, 3, 2)
    dV = c["Pm"].transpose(0, 1, 3, 2) @ dO
    dsc = c["Pm"] * (dPm - np.sum(dPm * c["Pm"], axis=-1, keepdims=True)) / np.sqrt(dh)
    dQ = _rope(dsc @ c["K"], c["cos"], c["sin"], inverse=True)
    dK = _rope(dsc.transpose(0, 1, 3, 2) @ c["Q"], c["cos"], c["sin"], inverse=True)

    def merge(t):
        return t.transpose(0, 2, 1, 3).reshape(batch * seq, d)

    dQ, dK, dV = merge(dQ), merge(dK), merge(dV)
    dWq, dWk, dWv = dQ.T @ c["Xn"], dK.T @ c["Xn"], dV.T @ c["Xn"]
    dXn = dQ @ Wq + dK @ Wk + dV @ Wv
    dX_branch, dg_attn = rmsnorm_bwd(dXn, c["N"], c["rstd"], g_attn)
    return dX_branch, dict(dWq=dWq, dWk=dWk, dWv=dWv, dWo=dWo, dg_attn=dg_attn)


def block_fwd_full(X, p, heads, batch, seq, eps=1e-6, dtype=np.float64):
    """Standard forward of one block: H = X + MHA(norm(X)); Out = H + FFN(norm(H))."""
    X = _f(X, dtype)
    M, cache = mha_fwd(X, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"], heads, batch, seq, eps, dtype)
    H = X + M
    U, _, _ = rmsnorm_fwd(H, p["g_ffn"], eps, dtype)
    _, _, _, Y = ffn_fwd_recompute(U, p["Wg"], p["Wu"], p["Wd"], dtype)
    return H + Y, H, cache


def block_bwd_full(X, dOut, p, heads, batch, seq, eps=1e-6):
    """Standard-mode backward (Alg. 3, first branch): exact gradients of everything."""
    _, H, cache = block_fwd_full(X, p, heads, batch, seq, eps)
    ffn = block_bwd_skip_exact_wgrad(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], eps)
    dH = ffn["dX"]
    dX_branch, mha = mha_bwd(dH, cache, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"])
    out = dict(dX=dH + dX_branch, dH=dH, dX_branch=dX_branch, dg_ffn=ffn["dgamma"],
               dWg=ffn["dWg"], dWu=ffn["dWu"], dWd=ffn["dWd"])
    out.update(mha)
    return out


# ------------------------------------------------ gradient averaging and optimizer step (Alg. 1)
def masked_grad_average(grads, contributes):
    """Eq. (1): mean of the per-rank gradients over the ranks that contribute (for q, k, v, o: the
    ranks that are neither failed nor neighbors; for the FFN matrices: every rank).  With no
    contributing rank the paper leaves the result open; the reading here is a zero gradient."""
    grads = [np.asarray(g, dtype=np.float64) for g in grads]
    idx = [i for i, c in enumerate(contributes) if c]
    if not idx:
        return np.zeros_like(grads[0])
    acc = np.zeros_like(grads[0])
    for i in idx:
        acc = acc + grads[i]
    return acc / len(idx)


def adamw_step(w, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One AdamW update with decoupled weight decay (the optimizer of the paper's training
    configuration); t counts from 1.  Returns the new (w, m, v)."""
    w, g, m, v = (np.asarray(x, dtype=np.float64) for x in (w, g, m, v))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    w = w * (1.0 - lr * weight_decay) - lr * mhat / (np.sqrt(vhat) + eps)
    return w, m, v


# ------------------------------------------------ token-stack harness (inputs only)
def stack_forward(ids, params, heads, eps=1e-6, dtype=np.float64, keep_last=None):
    """Embedding -> L blocks; returns the stored FFN inputs H_l and the last block's output.

    This only manufactures realistic inputs (H_l, and through the loss dOut_L) for the
    path under test, so callers may run it in float32 for speed and keep only the
    last `keep_last` H_l; the degraded backward itself is always checked in fp64."""
    batch, seq = ids.shape
    X = _f(params["emb"][ids.reshape(-1)], dtype)
    Hs = []
    L = len(params["blocks"])
    for li, p in enumerate(params["blocks"]):
        X, H, _ = block_fwd_full(X, p, heads, batch, seq, eps, dtype)
        Hs.append(H if keep_last is None or li >= L - keep_last else None)
    return Hs, X


def next_token_loss_grad(X_last, params, ids, eps=1e-6):
    """Summed next-token cross-entropy through final norm + untied LM head; returns (loss, dX_last)."""
    batch, seq = ids.shape
    Xn, N, rstd = rmsnorm_fwd(X_last, params["g_final"], eps)
    Wl = _f(params["lm_head"], np.float64)
    logits = Xn @ Wl.T
    logits -= logits.max(axis=1, keepdims=True)
    prob = np.exp(logits)
    prob /= prob.sum(axis=1, keepdims=True)
    tgt = np.roll(ids, -1, axis=1).reshape(-1)
    valid = np.ones((batch, seq), dtype=bool)
    valid[:, -1] = False
    valid = valid.reshape(-1)
    rows = np.arange(batch * seq)
    loss = -np.sum(np.log(prob[rows, tgt])[valid])
    dlog = prob
    dlog[rows, tgt] -= 1.0
    dlog[~valid] = 0.0
    dXn = dlog @ Wl
    dX, _ = rmsnorm_bwd(dXn, N, rstd, params["g_final"])
    return loss, dX
