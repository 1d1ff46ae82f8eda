"""GPU checks of the projection refresh (Alg. 3: V1 = top-r right singular vectors of the current
weights, Sec. 3.4) against the definition: numpy's SVD through the oracle's projection_from_svd,
or the singular subspace known by construction for planted spectra.

A singular basis is unique only up to a rotation inside the subspace (and only if s_r > s_{r+1}),
so what is compared is the subspace: the largest principal-angle sine between span(P_gpu) and
span(V1), plus P^T P = I.  The method is an iteration: with start error tan(theta0) the error
after q rounds is about (s_{r+1}/s_r)^(2q) tan(theta0) plus the rounding floor of the storage type
(bf16: entries of P carry 2^-9 relative error; the rounding of W moves its own singular
subspace by about ||W - bf16(W)|| / (s_r - s_{r+1})); the gates below are set from that.
"""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O
from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I
from gpu_util import dev, host, tdtype, up8, poisoned_ws

pytestmark = pytest.mark.gpu


def max_principal_sine(P, V):
    """sin of the largest principal angle between span(P) and span(V) (V orthonormal)."""
    Q, _ = np.linalg.qr(np.asarray(P, dtype=np.float64))
    s = np.linalg.svd(np.asarray(V, dtype=np.float64).T @ Q, compute_uv=False)
    return float(np.sqrt(max(0.0, 1.0 - min(s) ** 2)))


def refresh(W, V0, r, dtype, left=0, iters=8, cond=8, polish=5, pad=0):
    m, n = W.shape
    dim = m if left else n
    ldw = (up8(n) if dtype == "bf16" else n) + pad
    ldv = (up8(r) if dtype == "bf16" else r) + pad
    Wd, Vd = dev(W, dtype, ldw), dev(V0, dtype, ldv)
    Pd = torch.full((dim, ldv), float("nan"), dtype=tdtype(dtype), device="cuda")
    dt = B.BF16 if dtype == "bf16" else B.F32
    ws = poisoned_ws(B.mecefo_projection_workspace_bytes(dt, m, n, r, left))
    B.mecefo_projection_refresh(dt, Wd, m, n, ldw, left, Vd, ldv, r, iters, cond, polish, Pd, ldv, ws)
    torch.cuda.synchronize()
    P = host(Pd, r)
    assert np.all(np.isfinite(P))
    return P


def gaussian_start(seed, dim, r):
    return np.random.default_rng([77, seed]).standard_normal((dim, r)).astype(np.float32)


def orth_defect(P):
    P = np.asarray(P, dtype=np.float64)
    return float(np.linalg.norm(P.T @ P - np.eye(P.shape[1]), 2))


@pytest.mark.parametrize("m,n,r,left", [(96, 64, 16, 0), (130, 75, 9, 0), (64, 200, 20, 0), (96, 64, 16, 1), (75, 130, 9, 1)])
def test_refresh_f32_planted_gap(m, n, r, left):
    rng = np.random.default_rng([1, m, n, r])
    W, U, V = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(min(m, n), r), "f32")
    side = O.SIDE_OUTPUT if left else O.SIDE_INPUT
    want = O.projection_from_svd(W.astype(np.float64), r, side)
    P = refresh(W, gaussian_start(1, m if left else n, r), r, "f32", left=left, iters=10)
    sine = max_principal_sine(P, want)
    print("f32", m, n, r, left, "sin", sine, "orth", orth_defect(P))
    assert sine < 1e-3            # 0.5^(2*10) tan(theta0) is below 1e-4 for any reasonable start
    assert orth_defect(P) < 1e-4


@pytest.mark.parametrize("m,n,r,left,pad", [(1376, 512, 128, 0, 0), (512, 1376, 128, 0, 8), (1376, 512, 100, 1, 0), (344, 128, 33, 0, 8)])
def test_refresh_bf16_planted_gap(m, n, r, left, pad):
    rng = np.random.default_rng([2, m, n, r])
    W, U, V = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(min(m, n), r), "bf16")
    side = O.SIDE_OUTPUT if left else O.SIDE_INPUT
    want = O.projection_from_svd(W.astype(np.float64), r, side)
    P = refresh(W, gaussian_start(2, m if left else n, r), r, "bf16", left=left, iters=8, pad=pad)
    sine = max_principal_sine(P, want)
    print("bf16", m, n, r, left, "sin", sine, "orth", orth_defect(P))
    assert sine < 1e-2            # bf16 floor: rounding of W (its own subspace moves) and of P, about 2e-3 here
    assert orth_defect(P) < 1e-2


def test_light_settings_reach_the_bf16_floor():
    """Eight conditioning steps per round (s_1/s_r = 13 here: log(13^2)/log(3.44) + 3 = 7.2) and three
    polishing steps: the settings bench.py times."""
    rng = np.random.default_rng(8)
    m, n, r = 1376, 512, 128
    W, _, _ = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(n, r), "bf16")
    want = O.projection_from_svd(W.astype(np.float64), r)
    P = refresh(W, gaussian_start(8, n, r), r, "bf16", iters=8, cond=8, polish=3)
    sine, orth = max_principal_sine(P, want), orth_defect(P)
    print("light settings: sin", sine, "orth", orth)
    assert sine < 1e-2 and orth < 1e-2


def test_warm_start_needs_few_rounds():
    """Alg. 3 refreshes every tau steps from slowly moving weights: starting from the previous
    projection, two rounds recover the new subspace to the accuracy a cold start needs eight for."""
    rng = np.random.default_rng(3)
    m, n, r = 688, 256, 64
    W0, _, _ = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(n, r), "bf16")
    drift = I.round_to_bf16_grid((W0 + 0.002 * rng.standard_normal((m, n))).astype(np.float32))
    P_prev = O.projection_from_svd(W0.astype(np.float64), r).astype(np.float32)
    want = O.projection_from_svd(drift.astype(np.float64), r)
    before = max_principal_sine(P_prev, want)
    P = refresh(drift, P_prev, r, "bf16", iters=2)
    after = max_principal_sine(P, want)
    print("warm start: before", before, "after", after)
    assert after < 1e-2 and after < before / 10


def test_refreshed_projection_in_eq2_matches_svd_projection():
    """Eq. (2) with the refreshed P against Eq. (2) with the SVD's V1 (both through the oracle):
    dW depends on P only through the projector P P^T."""
    rng = np.random.default_rng(4)
    m, n, r, b = 344, 128, 32, 200
    W, _, _ = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(n, r), "bf16")
    P = refresh(W, gaussian_start(4, n, r), r, "bf16", iters=8)
    V1 = O.projection_from_svd(W.astype(np.float64), r)
    Gy, X = rng.standard_normal((b, m)), rng.standard_normal((b, n))
    a = O.wgrad_lowrank(Gy, X, P.astype(np.float64))
    bb = O.wgrad_lowrank(Gy, X, V1)
    rel = np.linalg.norm(a - bb) / np.linalg.norm(bb)
    print("Eq. (2) with refreshed vs SVD projection:", rel)
    assert rel < 1e-2


def test_no_gap_spectrum_captures_the_top_r_energy():
    """Gaussian weights have no spectral gap, so the boundary directions are not unique; what the
    method needs is the energy of the top-r subspace: ||W P||_F^2 >= (1 - eps) sum_{i<=r} s_i^2."""
    rng = np.random.default_rng(5)
    m, n, r = 1376, 512, 128
    W = I.ffn_weights(rng, n, m, "bf16")[0]          # [m x n] ~ N(0, 0.02^2)
    P = refresh(W, gaussian_start(5, n, r), r, "bf16", iters=8)
    s = np.linalg.svd(W.astype(np.float64), compute_uv=False)
    Q, _ = np.linalg.qr(P.astype(np.float64))
    got = np.linalg.norm(W.astype(np.float64) @ Q) ** 2
    best = float(np.sum(s[:r] ** 2))
    print("captured energy / optimum:", got / best, "orth", orth_defect(P))
    assert got <= best * (1 + 1e-9)
    assert got >= 0.98 * best
    assert orth_defect(P) < 1e-2


def test_refreshed_projection_on_gap_free_weights_captures_the_same_gradient_energy():
    """Config-shaped weights (C2 layer: d = 512, f = 1376, r = 128, N(0, 0.02^2): no spectral gap) have no unique
    top-r basis, so Eq. (2) with the refreshed projection and Eq. (2) with the oracle's SVD projection are
    different matrices.  What both must agree on is invariant to the choice of basis: the share of the exact
    gradient's energy that the projector keeps, ||dW_lr||_F^2 / ||dW*||_F^2 with dW_lr = dW* P P^T.  The GPU
    runs the whole chain (refresh from Gaussian noise, then mecefo_ffn_bwd_lowrank with its own P); the oracle
    takes numpy's SVD.  Gate: the two shares differ by less than 5 % of their value for every matrix (the
    refreshed basis holds >= 98 % of the top-r energy of W; measured difference about 1 %)."""
    from gpu_util import Layer, TOL, relerr
    d, f, r, b = 512, 1376, 128, 1024
    rng = np.random.default_rng(8)
    Wg, Wu, Wd, gamma = I.ffn_weights(rng, d, f, "bf16")
    U, dY = I.gaussian_block_io(rng, b, d, "bf16")
    P_gpu = [I.round_to_bf16_grid(refresh(W, gaussian_start(80 + i, W.shape[1], r), r, "bf16", iters=8))
             for i, W in enumerate((Wg, Wu, Wd))]
    P_svd = [O.projection_from_svd(W, r) for W in (Wg, Wu, Wd)]
    lay = Layer(b, d, f, "bf16", Wg, Wu, Wd, None, *P_gpu)
    dU = torch.empty(b, lay.ld_act_d, dtype=torch.bfloat16, device="cuda")
    B.mecefo_ffn_bwd_lowrank(lay.desc, lay.act(U), lay.act(dY), lay.Wg, lay.Wu, lay.Wd, *lay.projs(), B.SIDE_INPUT,
                             dU, lay.dWg, lay.dWu, lay.dWd, 0, lay.ws)
    torch.cuda.synchronize()
    got = lay.results()
    exact = O.ffn_bwd_exact(U, dY, Wg, Wu, Wd)
    with_gpu_p = O.ffn_bwd_lowrank(U, dY, Wg, Wu, Wd, *P_gpu)
    with_svd_p = O.ffn_bwd_lowrank(U, dY, Wg, Wu, Wd, *P_svd)
    for k in ("dWg", "dWu", "dWd"):
        assert relerr(got[k], with_gpu_p[k]) <= TOL["bf16"], k          # the usual parity, P as data
        e_gpu = np.linalg.norm(got[k]) ** 2 / np.linalg.norm(exact[k]) ** 2
        e_svd = np.linalg.norm(with_svd_p[k]) ** 2 / np.linalg.norm(exact[k]) ** 2
        print(k, "captured gradient energy: refreshed P", e_gpu, "SVD P", e_svd)
        assert abs(e_gpu - e_svd) <= 5e-2 * e_svd, (k, e_gpu, e_svd)


def test_zero_rounds_only_orthonormalises_the_start():
    rng = np.random.default_rng(6)
    m, n, r = 200, 96, 24
    W = rng.standard_normal((m, n)).astype(np.float32)
    V0 = gaussian_start(6, n, r)
    P = refresh(W, V0, r, "f32", iters=0, cond=6, polish=5)
    Q, _ = np.linalg.qr(V0.astype(np.float64))
    assert max_principal_sine(P, Q) < 1e-4      # same span as the start
    assert orth_defect(P) < 1e-4


def test_full_size_down_projection_subspace_known_by_construction():
    """C5's down projection shape (W_down [4096 x 11008], r = 1024, basis in R^11008): the host SVD
    of this size takes minutes, so the spectrum is planted and the subspace is known by construction."""
    rng = np.random.default_rng(7)
    m, n, r = 4096, 11008, 1024
    W, U, V = I.planted_spectrum_matrix(rng, m, n, I.spectrum_with_gap(m, r, decay=0.9995), "bf16")
    P = refresh(W, gaussian_start(7, n, r), r, "bf16", iters=8)
    sine = max_principal_sine(P, V[:, :r])
    print("C5 down projection: sin", sine, "orth", orth_defect(P))
    assert sine < 1e-2
    assert orth_defect(P) < 1e-2
