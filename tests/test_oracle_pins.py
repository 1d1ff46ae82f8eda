"""Pins of the CPU oracle against things other than itself.

The paper (arxiv 2510.16415) prints no numeric example for one layer, so the oracle
is pinned by: central finite differences of a scalar loss on a tiny block, an
independently written torch.autograd module (fp64, CPU), the full-rank identity of
Eq. (2), projector algebra, the Eckart-Young closed form for the SVD projection,
and invariants (linearity in dOut, RMSNorm scale invariance, the skip identity).
"""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O

EPS = 1e-6


def relerr(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


def tiny(seed=0, b=6, d=8, f=12, heads=2, batch=2, seq=3, std=0.5):
    rng = np.random.default_rng(seed)
    assert batch * seq == b
    p = dict(
        Wq=rng.standard_normal((d, d)) * std, Wk=rng.standard_normal((d, d)) * std,
        Wv=rng.standard_normal((d, d)) * std, Wo=rng.standard_normal((d, d)) * std,
        g_attn=1 + 0.2 * rng.standard_normal(d),
        Wg=rng.standard_normal((f, d)) * std, Wu=rng.standard_normal((f, d)) * std,
        Wd=rng.standard_normal((d, f)) * std, g_ffn=1 + 0.2 * rng.standard_normal(d))
    X = rng.standard_normal((b, d))
    dOut = rng.standard_normal((b, d))
    return p, X, dOut, heads, batch, seq


def fd_grad(fun, x, h=1e-6):
    """Central differences of scalar fun with respect to every entry of x (in place)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = fun()
        x[i] = old - h
        fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


# ---------------------------------------------------------------- finite differences
def test_fd_full_block_all_gradients():
    """Standard-mode backward (with MHA) equals finite differences of L = <dOut, Out>."""
    p, X, dOut, heads, batch, seq = tiny(1)
    g = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)

    def loss():
        out, _, _ = O.block_fwd_full(X, p, heads, batch, seq, EPS)
        return float(np.sum(out * dOut))

    assert relerr(g["dX"], fd_grad(loss, X)) < 1e-6
    for name, key in [("dWq", "Wq"), ("dWk", "Wk"), ("dWv", "Wv"), ("dWo", "Wo"),
                      ("dWg", "Wg"), ("dWu", "Wu"), ("dWd", "Wd"),
                      ("dg_attn", "g_attn"), ("dg_ffn", "g_ffn")]:
        assert relerr(g[name], fd_grad(loss, p[key])) < 1e-6, name


def test_fd_degraded_dx_and_exact_wgrad_with_frozen_attention():
    """With the attention output frozen to a constant c (H = X + c), finite differences of
    X -> H + FFN(norm(H)) give the degraded dX; those w.r.t. Wg, Wu, Wd, gamma give the
    exact FFN gradients that Eq. (2) approximates."""
    p, X, dOut, heads, batch, seq = tiny(2)
    M, _ = O.mha_fwd(X, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"], heads, batch, seq, EPS)
    c = M.copy()

    def loss():
        H = X + c
        U, _, _ = O.rmsnorm_fwd(H, p["g_ffn"], EPS)
        _, _, _, Y = O.ffn_fwd_recompute(U, p["Wg"], p["Wu"], p["Wd"])
        return float(np.sum((H + Y) * dOut))

    H = X + c
    r = 3
    Pg = O.projection_from_svd(p["Wg"], r)
    Pu = O.projection_from_svd(p["Wu"], r)
    Pd = O.projection_from_svd(p["Wd"], r)
    deg = O.block_bwd_skip(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], Pg, Pu, Pd, EPS)
    ex = O.block_bwd_skip_exact_wgrad(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], EPS)
    assert relerr(deg["dX"], fd_grad(loss, X)) < 1e-6
    assert relerr(deg["dgamma"], fd_grad(loss, p["g_ffn"])) < 1e-6
    fdg = {k: fd_grad(loss, p[k]) for k in ("Wg", "Wu", "Wd")}
    for k in ("Wg", "Wu", "Wd"):
        assert relerr(ex["d" + k], fdg[k]) < 1e-6
    # Eq. (2): the low-rank gradient is the exact one times the projector V1 V1^T
    for k, P in (("Wg", Pg), ("Wu", Pu), ("Wd", Pd)):
        assert relerr(deg["d" + k], fdg[k] @ P @ P.T) < 1e-6


def test_fd_no_norm_variant():
    """gamma=None means the stored tensor is fed to the FFN as is (U = H)."""
    rng = np.random.default_rng(3)
    b, d, f = 5, 6, 9
    H, dOut = rng.standard_normal((b, d)), rng.standard_normal((b, d))
    Wg, Wu, Wd = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    I_d, I_f = np.eye(d), np.eye(f)
    g = O.block_bwd_skip(H, dOut, None, Wg, Wu, Wd, I_d, I_d, I_f)

    def loss():
        _, _, _, Y = O.ffn_fwd_recompute(H, Wg, Wu, Wd)
        return float(np.sum((H + Y) * dOut))

    assert g["dgamma"] is None
    assert relerr(g["dX"], fd_grad(loss, H)) < 1e-6
    assert relerr(g["dWd"], fd_grad(loss, Wd)) < 1e-6


def test_fd_token_stack_loss_gradient():
    """Harness: summed next-token cross-entropy through final norm and LM head."""
    rng = np.random.default_rng(4)
    batch, seq, d, V = 2, 4, 6, 11
    ids = rng.integers(0, V, size=(batch, seq))
    params = dict(g_final=1 + 0.1 * rng.standard_normal(d), lm_head=rng.standard_normal((V, d)))
    X = rng.standard_normal((batch * seq, d))
    _, dX = O.next_token_loss_grad(X, params, ids, EPS)
    fd = fd_grad(lambda: O.next_token_loss_grad(X, params, ids, EPS)[0], X)
    assert relerr(dX, fd) < 1e-6
    # positions with no next token get no gradient
    assert np.all(dX.reshape(batch, seq, d)[:, -1] == 0)


# ------------------------------------------------------------- library cross-check
class _TorchBlock(torch.nn.Module):
    """LLaMA block written with torch ops only (independent of the oracle's numpy code)."""

    def __init__(self, p, heads, batch, seq):
        super().__init__()
        for k, v in p.items():
            setattr(self, k, torch.nn.Parameter(torch.tensor(v, dtype=torch.float64)))
        self.heads, self.batch, self.seq = heads, batch, seq

    @staticmethod
    def norm(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + EPS) * g

    def rope(self, t):
        dh = t.shape[-1]
        pos = torch.arange(self.seq, dtype=torch.float64)
        inv = 10000.0 ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
        ang = torch.outer(pos, inv)
        cos, sin = torch.cos(ang), torch.sin(ang)
        a, bb = t[..., : dh // 2], t[..., dh // 2:]
        return torch.cat([a * cos - bb * sin, a * sin + bb * cos], -1)

    def attn(self, X):
        B, S, h = self.batch, self.seq, self.heads
        d = X.shape[1]
        xn = self.norm(X, self.g_attn)
        sp = lambda t: t.view(B, S, h, d // h).transpose(1, 2)
        q, k, v = sp(xn @ self.Wq.T), sp(xn @ self.Wk.T), sp(xn @ self.Wv.T)
        o = torch.nn.functional.scaled_dot_product_attention(self.rope(q), self.rope(k), v, is_causal=True)
        return o.transpose(1, 2).reshape(B * S, d) @ self.Wo.T

    def ffn(self, H):
        u = self.norm(H, self.g_ffn)
        return (torch.nn.functional.silu(u @ self.Wg.T) * (u @ self.Wu.T)) @ self.Wd.T

    def forward(self, X, detach_attention=False):
        m = self.attn(X)
        H = X + (m.detach() if detach_attention else m)
        return H + self.ffn(H), H


def test_autograd_full_block_matches_oracle():
    p, X, dOut, heads, batch, seq = tiny(5, b=8, d=8, f=12, heads=2, batch=2, seq=4)
    blk = _TorchBlock(p, heads, batch, seq)
    Xt = torch.tensor(X, requires_grad=True)
    out, H = blk(Xt)
    (out * torch.tensor(dOut)).sum().backward()
    g = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)
    o_out, o_H, _ = O.block_fwd_full(X, p, heads, batch, seq, EPS)
    assert relerr(o_out, out.detach().numpy()) < 1e-12
    assert relerr(o_H, H.detach().numpy()) < 1e-12
    assert relerr(g["dX"], Xt.grad.numpy()) < 1e-10
    for name, key in [("dWq", "Wq"), ("dWk", "Wk"), ("dWv", "Wv"), ("dWo", "Wo"), ("dWg", "Wg"),
                      ("dWu", "Wu"), ("dWd", "Wd"), ("dg_attn", "g_attn"), ("dg_ffn", "g_ffn")]:
        assert relerr(g[name], getattr(blk, key).grad.numpy()) < 1e-10, name


def test_autograd_detached_attention_is_the_skip_backward():
    """Cutting the attention branch out of the autograd graph (forward unchanged) is the
    paper's backward-only skip: dX and the exact FFN gradients must match, and every MHA
    parameter must receive no gradient at all."""
    p, X, dOut, heads, batch, seq = tiny(6, b=8, d=8, f=12, heads=2, batch=2, seq=4)
    blk = _TorchBlock(p, heads, batch, seq)
    Xt = torch.tensor(X, requires_grad=True)
    out, H = blk(Xt, detach_attention=True)
    (out * torch.tensor(dOut)).sum().backward()
    ex = O.block_bwd_skip_exact_wgrad(H.detach().numpy(), dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], EPS)
    assert relerr(ex["dX"], Xt.grad.numpy()) < 1e-10
    assert relerr(ex["dgamma"], blk.g_ffn.grad.numpy()) < 1e-10
    for k in ("Wg", "Wu", "Wd"):
        assert relerr(ex["d" + k], getattr(blk, k).grad.numpy()) < 1e-10
    for k in ("Wq", "Wk", "Wv", "Wo", "g_attn"):
        assert getattr(blk, k).grad is None


# ------------------------------------------------------------------ Eq. (2) algebra
@pytest.mark.parametrize("side", [O.SIDE_INPUT, O.SIDE_OUTPUT])
def test_full_rank_identity(side):
    """r = projected dimension and P square orthonormal  =>  low-rank == exact."""
    rng = np.random.default_rng(7)
    b, m, n = 20, 9, 7
    Gy, X = rng.standard_normal((b, m)), rng.standard_normal((b, n))
    dim = n if side == O.SIDE_INPUT else m
    Q, _ = np.linalg.qr(rng.standard_normal((dim, dim)))
    assert relerr(O.wgrad_lowrank(Gy, X, Q, side), Gy.T @ X) < 1e-12


def test_full_rank_identity_whole_block():
    p, X, dOut, heads, batch, seq = tiny(8)
    d, f = p["Wg"].shape[1], p["Wg"].shape[0]
    H = X
    Pg = O.projection_from_svd(p["Wg"], d)      # gate/up project the d-dim input
    Pu = O.projection_from_svd(p["Wu"], d)
    rng = np.random.default_rng(80)
    Pd, _ = np.linalg.qr(rng.standard_normal((f, f)))   # down projects the f-dim input, r = d_ff
    lr = O.block_bwd_skip(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], Pg, Pu, Pd, EPS)
    ex = O.block_bwd_skip_exact_wgrad(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], EPS)
    for k in ("dX", "dgamma", "dWg", "dWu", "dWd"):
        assert relerr(lr[k], ex[k]) < 1e-12, k


def test_projector_algebra():
    rng = np.random.default_rng(9)
    b, m, n, r = 40, 11, 13, 4
    Gy, X = rng.standard_normal((b, m)), rng.standard_normal((b, n))
    W = rng.standard_normal((m, n))
    P = O.projection_from_svd(W, r)
    exact = Gy.T @ X
    lr = O.wgrad_lowrank(Gy, X, P)
    assert relerr(lr, exact @ P @ P.T) < 1e-12                    # associativity
    assert relerr(lr @ P, exact @ P) < 1e-12                      # agrees on the subspace
    assert np.linalg.matrix_rank(lr) <= r
    assert np.linalg.norm(lr) <= np.linalg.norm(exact) * (1 + 1e-12)
    assert relerr(lr @ P @ P.T, lr) < 1e-12                       # idempotent
    Q = O.projection_from_svd(W, r, O.SIDE_OUTPUT)
    lo = O.wgrad_lowrank(Gy, X, Q, O.SIDE_OUTPUT)
    assert relerr(lo, Q @ Q.T @ exact) < 1e-12
    # P need not be orthonormal: the formula is evaluated as written
    R = rng.standard_normal((n, r))
    assert relerr(O.wgrad_lowrank(Gy, X, R), exact @ R @ R.T) < 1e-12


def test_svd_projection_closed_forms():
    """V1 has orthonormal columns, spans the top-r eigenspace of W^T W (checked with a
    different LAPACK routine), and W V1 V1^T attains the Eckart-Young error."""
    rng = np.random.default_rng(10)
    m, n, r = 14, 10, 3
    W = rng.standard_normal((m, n))
    P = O.projection_from_svd(W, r)
    assert P.shape == (n, r)
    assert np.allclose(P.T @ P, np.eye(r), atol=1e-12)
    sig = np.linalg.svd(W, compute_uv=False)
    assert abs(np.linalg.norm(W - W @ P @ P.T) ** 2 - np.sum(sig[r:] ** 2)) < 1e-10
    _, vecs = np.linalg.eigh(W.T @ W)
    E = vecs[:, -r:]
    assert np.linalg.norm(P @ P.T - E @ E.T) < 1e-10
    Q = O.projection_from_svd(W, r, O.SIDE_OUTPUT)
    assert Q.shape == (m, r)
    assert abs(np.linalg.norm(W - Q @ Q.T @ W) ** 2 - np.sum(sig[r:] ** 2)) < 1e-10
    with pytest.raises(ValueError):
        O.projection_from_svd(W, n + 1)


def test_isotropic_error_closed_form():
    """Gaussian x independent of an orthonormal P: E|dW - dW_lr|^2 / |dW|^2 = 1 - r/n."""
    rng = np.random.default_rng(11)
    b, m, n, r = 4000, 24, 64, 16
    Gy, X = rng.standard_normal((b, m)), rng.standard_normal((b, n))
    P, _ = np.linalg.qr(rng.standard_normal((n, r)))
    ex = Gy.T @ X
    e = np.linalg.norm(ex - O.wgrad_lowrank(Gy, X, P)) ** 2 / np.linalg.norm(ex) ** 2
    assert abs(e - (1 - r / n)) < 0.04


# ------------------------------------------------------------------------ invariants
def test_skip_invariant():
    """Degraded dX is exactly dH; the full backward differs from it by exactly the
    attention branch's backward; the degraded result holds no MHA gradient."""
    p, X, dOut, heads, batch, seq = tiny(12)
    full = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)
    _, H, cache = O.block_fwd_full(X, p, heads, batch, seq, EPS)
    r = 4
    Ps = [O.projection_from_svd(p[k], r) for k in ("Wg", "Wu", "Wd")]
    deg = O.block_bwd_skip(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], *Ps, EPS)
    assert np.array_equal(deg["dX"], full["dH"])
    branch, _ = O.mha_bwd(full["dH"], cache, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"])
    assert relerr(full["dX"] - deg["dX"], branch) < 1e-12
    assert np.linalg.norm(branch) > 1e-3            # the dropped term is not trivially zero
    assert set(deg) == {"dX", "dgamma", "dWg", "dWu", "dWd"}


def test_linearity_in_upstream_gradient():
    p, X, dOut, *_ = tiny(13)
    Ps = [O.projection_from_svd(p[k], 3) for k in ("Wg", "Wu", "Wd")]
    args = (p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], *Ps, EPS)
    g1 = O.block_bwd_skip(X, dOut, *args)
    a = -2.5
    g2 = O.block_bwd_skip(X, a * dOut, *args)
    for k in g1:
        assert relerr(g2[k], a * g1[k]) < 1e-12
    g0 = O.block_bwd_skip(X, 0 * dOut, *args)
    for k in g0:
        assert np.all(g0[k] == 0)


def test_rmsnorm_scale_invariance():
    """With eps = 0 the norm ignores the scale of a row, so its input gradient is
    orthogonal to that row; and U has unit mean square when gamma = 1."""
    rng = np.random.default_rng(14)
    H, dU = rng.standard_normal((7, 16)), rng.standard_normal((7, 16))
    g = 1 + 0.3 * rng.standard_normal(16)
    U, N, rstd = O.rmsnorm_fwd(H, g, 0.0)
    dH, _ = O.rmsnorm_bwd(dU, N, rstd, g)
    assert np.max(np.abs(np.sum(dH * H, axis=1))) < 1e-12
    U1, _, _ = O.rmsnorm_fwd(H, np.ones(16), 0.0)
    assert np.allclose(np.mean(U1 * U1, axis=1), 1.0)
    U2, _, _ = O.rmsnorm_fwd(3.7 * H, g, 0.0)
    assert relerr(U2, U) < 1e-12


def test_swiglu_special_values():
    """silu(0)=0, silu'(0)=1/2; large |G| limits; A = silu(G)*Z against math.exp scalars."""
    import math
    U = np.eye(3)
    Wg = np.array([[0.0, 0, 0], [30.0, 0, 0], [-30.0, 0, 0]])     # G[0] = (0, 30, -30)
    Wu = np.array([[2.0, 0, 0], [2.0, 0, 0], [2.0, 0, 0]])
    G, Z, A, _ = O.ffn_fwd_recompute(U, Wg, Wu)
    assert A[0, 0] == 0 and abs(A[0, 1] - 60.0) < 1e-9 and abs(A[0, 2]) < 1e-10
    x = 0.7
    assert abs(O.ffn_fwd_recompute(np.array([[x]]), np.array([[1.0]]), np.array([[1.0]]))[2][0, 0]
               - x / (1 + math.exp(-x)) * x) < 1e-15
    # dG at G=0 is dA*Z/2
    Wd = np.eye(3)
    dY = np.array([[1.0, 1.0, 1.0], [0, 0, 0], [0, 0, 0]])
    _, dG, dZ = O.ffn_dgrad(dY, G, Z, Wg, Wu, Wd)
    assert abs(dG[0, 0] - 1.0) < 1e-15 and abs(dG[0, 1] - 2.0) < 1e-9 and abs(dG[0, 2]) < 1e-9
    assert dZ[0, 0] == 0


def test_flop_formula_of_eq2_matches_the_three_contractions():
    """Sec. 3.4 counts 2brn + 2brm + 2rmn for the chain; the three matmul shapes of
    wgrad_lowrank are exactly [b,n]x[n,r], [m,b]x[b,r], [m,r]x[r,n]."""
    b, m, n, r = 10, 6, 5, 2
    rng = np.random.default_rng(15)
    Gy, X, P = rng.standard_normal((b, m)), rng.standard_normal((b, n)), rng.standard_normal((n, r))
    T = X @ P
    C = Gy.T @ T
    assert T.shape == (b, r) and C.shape == (m, r) and (C @ P.T).shape == (m, n)
    assert 2 * b * r * n + 2 * b * r * m + 2 * r * m * n == 2 * (T.size * n + C.size * b + m * n * r)


def test_stack_forward_shapes_and_consistency():
    from paper_2510_16415_amd import inputs
    cfg = inputs.Config("T", 9, 16, 24, 2, 2, 5, 4, 2, "f32", stack=True)
    params = inputs.stack_params(cfg)
    # shrink the vocabulary tables for speed; ids stay inside the slice
    params["emb"], params["lm_head"] = params["emb"][:50], params["lm_head"][:50]
    ids = np.random.default_rng(0).integers(0, 50, size=(2, 5))
    Hs, X_last = O.stack_forward(ids, params, cfg.heads, EPS)
    assert len(Hs) == 2 and Hs[0].shape == (10, 16) and X_last.shape == (10, 16)
    # the last block's output is H + FFN(norm(H)) of its own stored H
    p = params["blocks"][-1]
    U, _, _ = O.rmsnorm_fwd(Hs[-1], p["g_ffn"], EPS)
    Y = O.ffn_fwd_recompute(U, p["Wg"], p["Wu"], p["Wd"])[3]
    assert relerr(Hs[-1] + Y, X_last) < 1e-12


def test_stack_forward_and_loss_gradient_match_a_torch_module_chain():
    """The harness that manufactures H_l and dOut for the stack configs (embedding lookup, L blocks,
    final norm, LM head, summed next-token cross-entropy) against the same model written with torch ops
    and differentiated by autograd: every stored H_l, the last block's output, the loss and its gradient
    with respect to the last block's output."""
    from paper_2510_16415_amd import inputs
    cfg = inputs.Config("T", 9, 16, 24, 2, 3, 5, 4, 2, "f32", stack=True)
    params = inputs.stack_params(cfg)
    V = 37
    params["emb"], params["lm_head"] = params["emb"][:V], params["lm_head"][:V]
    batch, seq = 2, 5
    ids = np.random.default_rng(3).integers(0, V, size=(batch, seq))
    Hs, X_last = O.stack_forward(ids, params, cfg.heads, EPS)
    loss, dX_last = O.next_token_loss_grad(X_last, params, ids, EPS)

    X = torch.tensor(np.asarray(params["emb"], dtype=np.float64))[torch.tensor(ids.reshape(-1))]
    t_H = []
    for p_l in params["blocks"]:
        blk = _TorchBlock({k: np.asarray(v, dtype=np.float64) for k, v in p_l.items()}, cfg.heads, batch, seq)
        X, H = blk(X)
        t_H.append(H.detach().numpy())
    Xl = X.detach().clone().requires_grad_(True)
    xn = _TorchBlock.norm(Xl, torch.tensor(np.asarray(params["g_final"], dtype=np.float64)))
    logits = (xn @ torch.tensor(np.asarray(params["lm_head"], dtype=np.float64)).T).view(batch, seq, V)
    tgt = torch.tensor(ids)[:, 1:].reshape(-1)
    t_loss = torch.nn.functional.cross_entropy(logits[:, :-1].reshape(-1, V), tgt, reduction="sum")
    t_loss.backward()
    assert len(Hs) == len(t_H) == cfg.layers
    for l, (a, b_) in enumerate(zip(Hs, t_H)):
        assert relerr(a, b_) < 1e-12, l
    assert relerr(X_last, X.detach().numpy()) < 1e-12
    assert abs(loss - t_loss.item()) < 1e-10 * abs(t_loss.item())
    assert relerr(dX_last, Xl.grad.numpy()) < 1e-10


def test_brute_force_index_sums_agree_with_the_numpy_oracle():
    """Brute force on tiny inputs: every output element of the neighbor-mode block backward written as an
    explicit index sum in pure Python (oracle/mecefo_loops.py, no numpy, no matrix routine) against the
    numpy oracle.  The two share no code; a transposed operand or a wrong index in either one fails here.
    Non-square everywhere (b != d != f, three different ranks) so that no transposition goes unnoticed."""
    from oracle import mecefo_loops as LO
    rng = np.random.default_rng(11)
    b, d, f = 5, 4, 7
    rg, ru, rd = 2, 3, 5
    H, dOut = rng.standard_normal((b, d)), rng.standard_normal((b, d))
    gamma = 1 + 0.2 * rng.standard_normal(d)
    Wg, Wu, Wd = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    Pg, Pu, Pd = rng.standard_normal((d, rg)), rng.standard_normal((d, ru)), rng.standard_normal((f, rd))
    want = O.block_bwd_skip(H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, EPS)
    got = LO.block_bwd_skip_loops(H.tolist(), dOut.tolist(), gamma.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist(),
                                  Pg.tolist(), Pu.tolist(), Pd.tolist(), EPS)
    for k in ("dX", "dgamma", "dWg", "dWu", "dWd"):
        assert np.asarray(got[k]).shape == want[k].shape, k
        assert relerr(np.asarray(got[k]), want[k]) < 1e-12, k


def test_saved_logsumexp_matches_library_routine_and_softmax():
    """The log-sum-exp that the forward keeps for the backward: checked against scipy's routine on
    the scaled, causally masked scores rebuilt from the cached Q and K, and exp(score - L) must
    give back the probabilities."""
    from scipy.special import logsumexp
    p, X, _, heads, batch, seq = tiny(11, b=10, d=8, f=12, heads=2, batch=2, seq=5)
    _, c = O.mha_fwd(X, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"], heads, batch, seq, EPS)
    dh = X.shape[1] // heads
    sc = np.einsum("bhqd,bhkd->bhqk", c["Q"], c["K"]) / np.sqrt(dh)
    for q in range(seq):
        ref = logsumexp(sc[:, :, q, : q + 1], axis=-1)
        assert np.allclose(c["L"][:, :, q], ref, rtol=1e-13, atol=1e-13)
        assert np.allclose(np.exp(sc[:, :, q, : q + 1] - c["L"][:, :, q, None]), c["Pm"][:, :, q, : q + 1], rtol=1e-12)
        assert np.all(c["Pm"][:, :, q, q + 1:] == 0)


def test_softmax_backward_row_term_equals_output_dot():
    """sum_k dP[q,k] P[q,k] = <dO[q], O[q]> per head (O = P V, dP = dO V^T): the identity that lets a
    backward pass work from the saved output instead of the probabilities."""
    p, X, dOut, heads, batch, seq = tiny(12, b=8, d=8, f=12, heads=2, batch=2, seq=4)
    _, c = O.mha_fwd(X, p["g_attn"], p["Wq"], p["Wk"], p["Wv"], p["Wo"], heads, batch, seq, EPS)
    d = X.shape[1]
    dh = d // heads
    dO = (dOut @ p["Wo"]).reshape(batch, seq, heads, dh).transpose(0, 2, 1, 3)
    dPm = dO @ c["V"].transpose(0, 1, 3, 2)
    lhs = np.sum(dPm * c["Pm"], axis=-1)
    Oh = c["O"].reshape(batch, seq, heads, dh).transpose(0, 2, 1, 3)
    rhs = np.sum(dO * Oh, axis=-1)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-13)


def test_masked_average_reduces_to_plain_mean_and_excludes_masked_ranks():
    """Eq. (1): with every rank contributing it is the plain mean; a masked rank's values (even
    non-finite ones) do not enter; the divisor is the number of contributing ranks."""
    rng = np.random.default_rng(13)
    G = [rng.standard_normal((5, 7)) for _ in range(4)]
    assert np.allclose(O.masked_grad_average(G, [1, 1, 1, 1]), np.mean(G, axis=0), rtol=1e-15)
    G[2][:] = np.nan
    got = O.masked_grad_average(G, [1, 1, 0, 1])
    assert np.allclose(got, (G[0] + G[1] + G[3]) / 3.0, rtol=1e-15)
    assert np.array_equal(O.masked_grad_average(G, [0, 0, 0, 0]), np.zeros((5, 7)))
    assert np.allclose(O.masked_grad_average(G, [0, 1, 0, 0]), G[1])


def test_adamw_matches_torch_optimizer():
    rng = np.random.default_rng(14)
    w0 = rng.standard_normal((6, 5))
    p = torch.nn.Parameter(torch.tensor(w0))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 5):
        g = rng.standard_normal((6, 5))
        p.grad = torch.tensor(g)
        opt.step()
        w, m, v = O.adamw_step(w, g, m, v, t, 3e-3)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14), t
