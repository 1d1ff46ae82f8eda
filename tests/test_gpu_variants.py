"""GPU parity of the tunable variants of the neighbor branch (the paper's extension paragraph:
skip on a subset, extra checkpoints, other ranks): mecefo_block_bwd_skip_ex."""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O
from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I
from gpu_util import TOL, Layer, assert_close, dev, host
from test_gpu_parity import make_case, oracle_block

pytestmark = pytest.mark.gpu
EPS = 1e-6


def run_ex(lay, c, G=None, Z=None, mask=0, drop_P=False):
    Hd, dOd = lay.act(c["H"]), lay.act(c["dOut"])
    dX = torch.full_like(dOd, float("nan"))
    Ps = [None if (drop_P and mask & (1 << i)) else p for i, p in enumerate(lay.projs())]
    B.mecefo_block_bwd_skip_ex(lay.desc, Hd, dOd, lay.gamma, lay.Wg, lay.Wu, lay.Wd, *Ps, lay.side, dX, lay.dgamma,
                               lay.dWg, lay.dWu, lay.dWd, 0, lay.ws, G=G, Z=Z, exact_wgrad_mask=mask)
    torch.cuda.synchronize()
    return lay.results(dX)


def layer_of(c, b, d, f, dtype):
    return Layer(b, d, f, dtype, c["Wg"], c["Wu"], c["Wd"], c["gamma"], c["Pg"], c["Pu"], c["Pd"], EPS)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_default_options_are_the_plain_call_bit_for_bit(dtype):
    b, d, f, r = 300, 128, 344, 24
    c = make_case(51, b, d, f, r, dtype)
    lay = layer_of(c, b, d, f, dtype)
    a = lay.block_bwd_skip(c["H"], c["dOut"])
    bb = run_ex(lay, c)
    for k in a:
        assert np.array_equal(a[k], bb[k]), k


@pytest.mark.parametrize("dtype,b,d,f,r", [("f32", 77, 48, 100, 12), ("bf16", 300, 128, 344, 24), ("bf16", 513, 256, 1000, 64)])
def test_extra_checkpoints_saved_gate_and_up(dtype, b, d, f, r):
    """With G and Z kept by the forward pass the result is the same backward without the recompute."""
    c = make_case(52, b, d, f, r, dtype)
    lay = layer_of(c, b, d, f, dtype)
    U, _, _ = O.rmsnorm_fwd(c["H"], c["gamma"], EPS)
    G, Z, _, _ = O.ffn_fwd_recompute(U, c["Wg"], c["Wu"])
    cast = I.round_to_bf16_grid if dtype == "bf16" else (lambda x: x)
    Gd, Zd = lay.act(cast(G.astype(np.float32)), wide=True), lay.act(cast(Z.astype(np.float32)), wide=True)
    got = run_ex(lay, c, G=Gd, Z=Zd)
    errs = assert_close(got, oracle_block(c), TOL[dtype], label="saved G, Z: ")
    print(dtype, errs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mask", [1, 2, 4, 5, 7])
def test_exact_wgrad_on_a_subset_of_the_matrices(dtype, mask):
    b, d, f, r = 260, 128, 344, 24
    c = make_case(53, b, d, f, r, dtype)
    lay = layer_of(c, b, d, f, dtype)
    want = oracle_block(c)
    exact = O.block_bwd_skip_exact_wgrad(c["H"], c["dOut"], c["gamma"], c["Wg"], c["Wu"], c["Wd"], EPS)
    for i, k in enumerate(("dWg", "dWu", "dWd")):
        if mask & (1 << i):
            want[k] = exact[k]
    got = run_ex(lay, c, mask=mask, drop_P=True)
    errs = assert_close(got, want, TOL[dtype], label=f"mask {mask}: ")
    print(dtype, mask, errs)


def test_mask_validation():
    b, d, f, r = 64, 64, 104, 8
    c = make_case(54, b, d, f, r, "bf16")
    lay = layer_of(c, b, d, f, "bf16")
    with pytest.raises(B.MecefoError):
        run_ex(lay, c, mask=8)
    with pytest.raises(B.MecefoError):           # a low-rank matrix still needs its projection
        run_ex(lay, c, mask=0, drop_P=False, G=lay.act(c["H"]))   # G without Z


def test_moe_expert_shaped_ffn_ragged_token_groups():
    """An expert of a mixture-of-experts block is the same SwiGLU FFN with a small d_ff, applied to the tokens
    routed to it (the paper's MLA + MoE variant, App. "other model structures"; expert sizes are not given, so
    the shape is a stand-in: d = 512, eight experts of d_ff = 200, r = 32 per matrix).  Each expert's token
    group goes through mecefo_ffn_bwd_lowrank: groups of very different sizes, one empty, one of a single
    token, one ragged against every tile; the routed groups partition the token batch, so the sum of the
    experts' input gradients scattered back must equal the oracle's, group by group."""
    d, f, r, experts = 512, 200, 32, 8
    sizes = [0, 1, 37, 256, 300, 64, 129, 513]
    rng = np.random.default_rng(61)
    total = sum(sizes)
    U, dY = I.gaussian_block_io(rng, total, d, "bf16")
    order = rng.permutation(total)                      # which tokens each expert received
    start = 0
    worst = {}
    for e in range(experts):
        idx = np.sort(order[start:start + sizes[e]])
        start += sizes[e]
        Wg, Wu, Wd, _ = I.ffn_weights(rng, d, f, "bf16")
        Ps = [I.random_orthonormal(rng, n, r, "bf16") for n in (d, d, f)]
        lay = Layer(sizes[e], d, f, "bf16", Wg, Wu, Wd, None, *Ps, EPS)
        Ue, dYe = U[idx], dY[idx]
        dU = torch.full((sizes[e], lay.ld_act_d), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.mecefo_ffn_bwd_lowrank(lay.desc, lay.act(Ue) if sizes[e] else None, lay.act(dYe) if sizes[e] else None,
                                 lay.Wg, lay.Wu, lay.Wd, *lay.projs(), B.SIDE_INPUT, dU if sizes[e] else None,
                                 lay.dWg, lay.dWu, lay.dWd, 0, lay.ws)
        torch.cuda.synchronize()
        got = lay.results()
        if sizes[e] == 0:
            for k in ("dWg", "dWu", "dWd"):
                assert np.array_equal(got[k], np.zeros_like(got[k])), (e, k)     # an expert nobody was routed to
            continue
        got["dU"] = host(dU, d)
        want = O.ffn_bwd_lowrank(Ue, dYe, Wg, Wu, Wd, *Ps)
        errs = assert_close(got, want, TOL["bf16"], keys=["dU", "dWg", "dWu", "dWd"], label=f"expert {e} ({sizes[e]} tokens): ")
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
    print("MoE-expert-shaped groups, worst errors", worst)
