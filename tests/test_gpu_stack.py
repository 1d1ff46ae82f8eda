"""GPU checks of what surrounds the hot path in Alg. 1 / Alg. 2: the neighbor-mode stack (forward
keeping only H_l, chained degraded backward), Eq. (1) gradient averaging over simulated ranks, the
AdamW step, and HIP-graph capture of a whole stack pass."""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O
from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I
from gpu_util import TOL, dev, host, relerr, tdtype, up8, poisoned_ws

pytestmark = pytest.mark.gpu
EPS = 1e-6


# ------------------------------------------------------------------ Eq. (1)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mask", [[1, 1, 1, 1], [1, 0, 1, 0], [0, 0, 1, 0], [0, 0, 0, 0]])
def test_grad_average_matches_eq1(dtype, mask):
    rng = np.random.default_rng([31, sum(mask)])
    n = 1000 * 37 + 3                      # not a multiple of the vector width
    G = [rng.standard_normal(n).astype(np.float32) for _ in range(4)]
    if dtype == "bf16":
        G = [I.round_to_bf16_grid(g) for g in G]
    t = tdtype(dtype)
    Gd = [torch.from_numpy(g).to(t).cuda() if m else None for g, m in zip(G, mask)]   # masked ranks pass NULL
    out = torch.full((n,), float("nan"), dtype=t, device="cuda")
    B.mecefo_grad_average(B.BF16 if dtype == "bf16" else B.F32, Gd, mask, out, n)
    torch.cuda.synchronize()
    want = O.masked_grad_average(G, mask)
    got = out.float().cpu().numpy()
    if sum(mask) == 0:
        assert np.array_equal(got, np.zeros(n, dtype=np.float32))
    else:
        assert relerr(got, want) < (1e-6 if dtype == "f32" else 4e-3)


def test_grad_average_in_place_on_the_first_rank():
    rng = np.random.default_rng(32)
    G = [rng.standard_normal(4096).astype(np.float32) for _ in range(3)]
    Gd = [torch.from_numpy(g).cuda() for g in G]
    B.mecefo_grad_average(B.F32, Gd, [1, 1, 1], Gd[0], 4096)
    torch.cuda.synchronize()
    assert relerr(Gd[0].cpu().numpy(), O.masked_grad_average(G, [1, 1, 1])) < 1e-6


# ------------------------------------------------------------------ AdamW
def f32(x):
    """The hyper-parameter value the C ABI receives (a float): the oracle is given the same number."""
    return float(np.float32(x))


HP = dict(beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), weight_decay=f32(0.01))


def test_adamw_f32_three_steps():
    rng = np.random.default_rng(33)
    n = 5003
    w = rng.standard_normal(n).astype(np.float32)
    Wd = torch.from_numpy(w.copy()).cuda()
    M = torch.zeros(n, device="cuda")
    V = torch.zeros(n, device="cuda")
    wo, mo, vo = w.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 4):
        g = rng.standard_normal(n).astype(np.float32)
        B.mecefo_adamw_step(B.F32, B.F32, Wd, torch.from_numpy(g).cuda(), M, V, n, t, 3e-3)
        wo, mo, vo = O.adamw_step(wo, g, mo, vo, t, f32(3e-3), **HP)
    torch.cuda.synchronize()
    assert relerr(Wd.cpu().numpy(), wo) < 1e-6
    assert relerr(M.cpu().numpy(), mo) < 1e-6 and relerr(V.cpu().numpy(), vo) < 1e-6


def test_adamw_bf16_weights_round_once_per_step():
    """bf16 parameters: every step is compared from the GPU's own (rounded) weights, so that both
    sides round the same update; the result must be the oracle's value within one bf16 ulp."""
    rng = np.random.default_rng(34)
    n = 4099
    w = I.round_to_bf16_grid(rng.standard_normal(n).astype(np.float32))
    Wd = torch.from_numpy(w).to(torch.bfloat16).cuda()
    M = torch.zeros(n, device="cuda")
    V = torch.zeros(n, device="cuda")
    for t in range(1, 4):
        g = rng.standard_normal(n).astype(np.float32)
        w_before = Wd.float().cpu().numpy().astype(np.float64)
        m_before, v_before = M.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64)
        B.mecefo_adamw_step(B.BF16, B.F32, Wd, torch.from_numpy(g).cuda(), M, V, n, t, 1e-2)
        torch.cuda.synchronize()
        wo, _, _ = O.adamw_step(w_before, g, m_before, v_before, t, f32(1e-2), **HP)
        got = Wd.float().cpu().numpy()
        assert np.all(np.abs(got - wo) <= np.abs(wo) * 2.0 ** -8 + 1e-30)


# ------------------------------------------------------------------ the stack
class Stack:
    def __init__(self, n_layers, batch, seq, d, f, heads, r, dtype, seed):
        rng = np.random.default_rng([35, seed])
        self.n_layers, self.dtype, self.heads, self.batch, self.seq = n_layers, dtype, heads, batch, seq
        self.b, self.d, self.f, self.r = batch * seq, d, f, r
        self.params = []
        for _ in range(n_layers):
            Wg, Wu, Wd, _ = I.ffn_weights(rng, d, f, dtype, std=0.05)
            Wq, Wk, Wv, Wo, _ = I.mha_weights(rng, d, dtype, std=1.0 / np.sqrt(d))
            p = dict(Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, Wg=Wg, Wu=Wu, Wd=Wd, g_attn=I.perturbed_gain(rng, d, dtype),
                     g_ffn=I.perturbed_gain(rng, d, dtype))
            p["P"] = [I.random_orthonormal(rng, d, r, dtype), I.random_orthonormal(rng, d, r, dtype),
                      I.random_orthonormal(rng, f, r, dtype)]
            self.params.append(p)
        self.X0, self.dOut = I.gaussian_block_io(rng, self.b, d, dtype)
        al = 8 if dtype == "bf16" else 1
        self.ldf = (f + al - 1) // al * al
        dt = B.BF16 if dtype == "bf16" else B.F32
        self.desc = B.make_desc(self.b, d, f, dt, B.F32, d, self.ldf, d, self.ldf, EPS)
        self.attn = B.make_attn_desc(batch, seq, heads, d)
        self.dev_layers = []
        for p in self.params:
            e = {k: dev(p[k], dtype) for k in ("g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu")}
            e["Wd"] = dev(p["Wd"], dtype, self.ldf)
            self.dev_layers.append(e)
        self.lw = B.layer_weights(self.dev_layers)
        t = tdtype(dtype)
        self.H = [torch.full((self.b, d), float("nan"), dtype=t, device="cuda") for _ in range(n_layers)]
        self.X0d, self.dOd = dev(self.X0, dtype), dev(self.dOut, dtype)
        self.Xout = torch.full((self.b, d), float("nan"), dtype=t, device="cuda")
        self.dX = torch.full((self.b, d), float("nan"), dtype=t, device="cuda")
        self.Pdev = [[dev(P, dtype, up8(r) if dtype == "bf16" else r) for P in p["P"]] for p in self.params]
        self.grads = [dict(dg_ffn=torch.full((d,), float("nan"), device="cuda"),
                           dWg=torch.full((f, d), float("nan"), device="cuda"),
                           dWu=torch.full((f, d), float("nan"), device="cuda"),
                           dWd=torch.full((d, self.ldf), float("nan"), device="cuda")) for _ in range(n_layers)]
        self.lr = B.layer_lowrank([dict(Pg=B.proj(P[0], r), Pu=B.proj(P[1], r), Pd=B.proj(P[2], r), **g)
                                   for P, g in zip(self.Pdev, self.grads)])
        self.ws = poisoned_ws(B.mecefo_stack_workspace_bytes(self.desc, self.attn, r, r, r))

    def forward(self):
        B.mecefo_stack_fwd_neighbor(self.desc, self.attn, self.lw, self.X0d, self.H, self.Xout, self.ws)

    def backward(self, accumulate=0):
        B.mecefo_stack_bwd_skip(self.desc, self.lw, self.H, self.lr, B.SIDE_INPUT, self.dOd, self.dX, accumulate, self.ws)

    def oracle(self):
        x = self.X0.astype(np.float64)
        Hs = []
        for p in self.params:
            x, H, _ = O.block_fwd_full(x, p, self.heads, self.batch, self.seq, EPS)
            Hs.append(H)
        g = self.dOut.astype(np.float64)
        res = [None] * self.n_layers
        for l in range(self.n_layers - 1, -1, -1):
            p = self.params[l]
            res[l] = O.block_bwd_skip(Hs[l], g, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], *p["P"], EPS)
            g = res[l]["dX"]
        return x, Hs, res

    def results(self):
        torch.cuda.synchronize()
        return dict(Xout=host(self.Xout), H=[host(h) for h in self.H], dX=host(self.dX),
                    grads=[dict(dgamma=host(g["dg_ffn"]), dWg=host(g["dWg"]), dWu=host(g["dWu"]),
                                dWd=host(g["dWd"], self.f)) for g in self.grads])


def _ffn_out(H, p):
    """Out = H + FFN(RMSNorm(H)) with the oracle, from a given stored tensor."""
    U, _, _ = O.rmsnorm_fwd(H, p["g_ffn"], EPS)
    return np.asarray(H, dtype=np.float64) + O.ffn_fwd_recompute(U, p["Wg"], p["Wu"], p["Wd"])[3]


@pytest.mark.parametrize("dtype,n_layers,batch,seq,d,f,heads,r", [("f32", 3, 2, 24, 32, 88, 4, 8),
                                                                  ("bf16", 4, 2, 128, 128, 344, 4, 32)])
def test_neighbor_mode_stack_forward_and_chained_backward(dtype, n_layers, batch, seq, d, f, heads, r):
    """Gated at the stated tolerance, layer by layer with teacher forcing: every stored H_l against the oracle
    applied to the GPU's own H_(l-1) (the FFN half of layer l-1 and the attention half of layer l: one block
    of arithmetic), the output against the oracle applied to the GPU's last H, and the top layer of the
    backward (its upstream gradient is an input).  The errors of the free-running chains (forward from X0,
    backward down to layer 0) are printed, not gated: the stack calls are the per-layer calls bit for bit
    (next test), and those are gated layer by layer with teacher forcing in test_gpu_parity.py."""
    st = Stack(n_layers, batch, seq, d, f, heads, r, dtype, 1)
    st.forward()
    st.backward()
    got = st.results()
    tol = TOL[dtype]
    x = st.X0.astype(np.float64)
    for l in range(n_layers):
        _, H_want, _ = O.block_fwd_full(x, st.params[l], heads, batch, seq, EPS)
        assert relerr(got["H"][l], H_want) <= tol, (l, relerr(got["H"][l], H_want))
        x = _ffn_out(got["H"][l], st.params[l])          # teacher forcing: continue from the GPU's stored tensor
    assert relerr(got["Xout"], x) <= tol
    top = n_layers - 1
    p = st.params[top]
    want_top = O.block_bwd_skip(got["H"][top], st.dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], *p["P"], EPS)
    for k in ("dgamma", "dWg", "dWu", "dWd"):
        assert relerr(got["grads"][top][k], want_top[k]) <= tol, (k, relerr(got["grads"][top][k], want_top[k]))
    if n_layers == 1:
        assert relerr(got["dX"], want_top["dX"]) <= tol
    xo, Hs, res = st.oracle()
    chain = {f"layer {l} {k}": relerr(got["grads"][l][k], res[l][k]) for l in range(n_layers) for k in ("dWg", "dWd")}
    print(dtype, "free-running (not gated): Xout", relerr(got["Xout"], xo), "H[last]", relerr(got["H"][-1], Hs[-1]),
          "dX", relerr(got["dX"], res[0]["dX"]), chain)
    assert all(np.isfinite(v) for v in chain.values())


def test_stack_calls_equal_the_per_layer_calls_bit_for_bit():
    st = Stack(3, 2, 64, 64, 172, 4, 16, "bf16", 2)
    st.forward()
    st.backward()
    a = st.results()
    # the same chain through the single-block entry points
    bws = poisoned_ws(B.mecefo_workspace_bytes(st.desc, st.r, st.r, st.r))
    g = st.dOd.clone()
    for l in range(2, -1, -1):
        e, P, G = st.dev_layers[l], st.Pdev[l], st.grads[l]
        for t in G.values():
            t.fill_(float("nan"))
        B.mecefo_block_bwd_skip(st.desc, st.H[l], g, e["g_ffn"], e["Wg"], e["Wu"], e["Wd"], B.proj(P[0], st.r),
                                B.proj(P[1], st.r), B.proj(P[2], st.r), B.SIDE_INPUT, g, G["dg_ffn"], G["dWg"], G["dWu"],
                                G["dWd"], 0, bws)
    torch.cuda.synchronize()
    assert np.array_equal(host(g), a["dX"])
    b = st.results()
    for l in range(3):
        for k in a["grads"][l]:
            assert np.array_equal(a["grads"][l][k], b["grads"][l][k]), (l, k)


def _mixed_setup(seed, modes):
    """A small bf16 stack whose layers are forwarded one by one in standard mode (everything a
    standard-mode backward needs is kept), plus gradient buffers filled with NaN canaries."""
    import ctypes as C
    n_layers = len(modes)
    st = Stack(n_layers, 2, 96, 128, 344, 4, 32, "bf16", seed)
    t = tdtype("bf16")
    act = lambda: torch.full((st.b, st.d), float("nan"), dtype=t, device="cuda")
    fws = poisoned_ws(B.mecefo_block_fwd_workspace_bytes(st.desc, st.attn))
    saved, x = [], st.X0d
    for l in range(n_layers):
        e = st.dev_layers[l]
        out = dict(Out=act(), H=act(), Q=act(), K=act(), V=act(), O=act(),
                   L=torch.full((st.batch * st.heads * st.seq,), float("nan"), device="cuda"))
        B.mecefo_block_fwd(st.desc, st.attn, dict(X=x, **e), out, fws)
        saved.append(dict(X=x, **{k: out[k] for k in ("H", "Q", "K", "V", "O", "L")}))
        x = out["Out"]
    torch.cuda.synchronize()
    nanf = lambda *shape: torch.full(shape, float("nan"), device="cuda")
    d, f = st.d, st.f
    grads = [dict(dg_attn=nanf(d), dg_ffn=nanf(d), dWq=nanf(d, d), dWk=nanf(d, d), dWv=nanf(d, d), dWo=nanf(d, d),
                  dWg=nanf(f, d), dWu=nanf(f, d), dWd=nanf(d, st.ldf)) for _ in range(n_layers)]
    inputs = [dict(dOut=st.dOd, **saved[l], **st.dev_layers[l]) for l in range(n_layers)]
    low = B.layer_lowrank([dict(Pg=B.proj(P[0], st.r), Pu=B.proj(P[1], st.r), Pd=B.proj(P[2], st.r),
                                dg_ffn=g["dg_ffn"], dWg=g["dWg"], dWu=g["dWu"], dWd=g["dWd"])
                           for P, g in zip(st.Pdev, grads)])
    ws = poisoned_ws(B.mecefo_stack_mixed_workspace_bytes(st.desc, st.attn, st.r, st.r, st.r))
    return st, inputs, grads, low, ws, C


def test_mixed_stack_standard_and_neighbor_layers():
    """The skip on a subset of the layers (Sec. 5, extension paragraph): layers 1 and 3 run in neighbor
    mode, layers 0 and 2 in standard mode.  The driver must equal the chain of per-layer calls bit for bit
    (those are gated against the oracle layer by layer elsewhere), a neighbor-mode layer must leave its
    MHA gradient buffers untouched, and the top layer (whose upstream gradient is an input) is compared
    with the oracle at the stated tolerance."""
    modes = [B.MODE_STANDARD, B.MODE_NEIGHBOR, B.MODE_STANDARD, B.MODE_NEIGHBOR]
    st, inputs, grads, low, ws, _ = _mixed_setup(11, modes)
    dX = torch.full((st.b, st.d), float("nan"), dtype=tdtype("bf16"), device="cuda")
    B.mecefo_stack_bwd_mixed(st.desc, st.attn, modes, inputs, [dict(dX=dX, **g) for g in grads], low, B.SIDE_INPUT,
                             None, None, st.dOd, dX, 0, ws)
    torch.cuda.synchronize()
    got = [{k: host(v) for k, v in g.items()} for g in grads]
    got_dX = host(dX)
    for l, m in enumerate(modes):
        for k in ("dg_attn", "dWq", "dWk", "dWv", "dWo"):
            if m == B.MODE_NEIGHBOR:
                assert np.all(np.isnan(got[l][k])), (l, k)          # Sec. 3.2: no MHA gradient from a neighbor-mode layer
            else:
                assert np.all(np.isfinite(got[l][k])), (l, k)
        for k in ("dg_ffn", "dWg", "dWu"):
            assert np.all(np.isfinite(got[l][k])), (l, k)
    # the same chain through the per-layer entry points
    g = st.dOd.clone()
    ref = [dict((k, torch.full_like(v, float("nan"))) for k, v in gr.items()) for gr in grads]
    for l in range(len(modes) - 1, -1, -1):
        e, P = st.dev_layers[l], st.Pdev[l]
        if modes[l] == B.MODE_NEIGHBOR:
            B.mecefo_block_bwd_skip(st.desc, inputs[l]["H"], g, e["g_ffn"], e["Wg"], e["Wu"], e["Wd"], B.proj(P[0], st.r),
                                    B.proj(P[1], st.r), B.proj(P[2], st.r), B.SIDE_INPUT, g, ref[l]["dg_ffn"],
                                    ref[l]["dWg"], ref[l]["dWu"], ref[l]["dWd"], 0, ws)
        else:
            B.mecefo_block_bwd_full(st.desc, st.attn, dict(inputs[l], dOut=g), dict(dX=g, **ref[l]), 0, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(g), got_dX)
    for l in range(len(modes)):
        for k, v in ref[l].items():
            assert np.array_equal(host(v), got[l][k], equal_nan=True), (l, k)
    top = len(modes) - 1
    p = st.params[top]
    want = O.block_bwd_skip(host(inputs[top]["H"]), st.dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], *p["P"], EPS)
    for k, kk in (("dg_ffn", "dgamma"), ("dWg", "dWg"), ("dWu", "dWu")):
        assert relerr(got[top][k], want[kk]) <= TOL["bf16"], (k, relerr(got[top][k], want[kk]))
    assert relerr(got[top]["dWd"][:, :st.f], want["dWd"]) <= TOL["bf16"]


def test_mixed_stack_refreshes_projections_when_the_counter_is_due():
    """Alg. 3's refresh branch wired into the driver: with tau = 10 and counters (0, 0, 0, 5) the neighbor-mode
    layer 1 (t = 0) recomputes its three projections before its backward, layer 3 (t = 5) reuses them; the
    standard-mode layers keep their counters; every neighbor-mode layer's counter grows by one."""
    modes = [B.MODE_STANDARD, B.MODE_NEIGHBOR, B.MODE_STANDARD, B.MODE_NEIGHBOR]
    st, inputs, grads, low, ws, C = _mixed_setup(12, modes)
    before = [[host(P) for P in layer] for layer in st.Pdev]
    # what the refresh of layer 1 must produce: the refresh call itself with the same arguments
    pol = B.RefreshPolicy(10, 2, 8, 3)
    e = st.dev_layers[1]
    expect = []
    for W, m, n, ldw, P in ((e["Wg"], st.f, st.d, st.d, st.Pdev[1][0]), (e["Wu"], st.f, st.d, st.d, st.Pdev[1][1]),
                            (e["Wd"], st.d, st.f, st.ldf, st.Pdev[1][2])):
        out = torch.empty_like(P)
        pws = poisoned_ws(B.mecefo_projection_workspace_bytes(B.BF16, m, n, st.r, 0))
        B.mecefo_projection_refresh(B.BF16, W, m, n, ldw, 0, P, P.stride(0), st.r, 2, 8, 3, out, out.stride(0), pws)
        expect.append(host(out))
    t = (C.c_int64 * 4)(0, 0, 0, 5)
    dX = torch.full((st.b, st.d), float("nan"), dtype=tdtype("bf16"), device="cuda")
    B.mecefo_stack_bwd_mixed(st.desc, st.attn, modes, inputs, [dict(dX=dX, **g) for g in grads], low, B.SIDE_INPUT,
                             pol, t, st.dOd, dX, 0, ws)
    torch.cuda.synchronize()
    assert list(t) == [0, 1, 0, 6]
    after = [[host(P) for P in layer] for layer in st.Pdev]
    for i in range(3):
        assert np.array_equal(after[3][i], before[3][i])              # not due: reused
        assert np.array_equal(after[0][i], before[0][i]) and np.array_equal(after[2][i], before[2][i])
        assert not np.array_equal(after[1][i], before[1][i])          # due: recomputed in place ...
        assert np.array_equal(after[1][i], expect[i])                 # ... by the refresh call, bit for bit
        Pn = after[1][i][:, :st.r].astype(np.float64)
        assert np.linalg.norm(Pn.T @ Pn - np.eye(st.r), 2) < 1e-2     # orthonormal basis (bf16 floor)
    # the gradients of layer 1 were formed with the refreshed projection
    p = st.params[1]
    H1 = host(inputs[1]["H"])
    assert np.all(np.isfinite(host(grads[1]["dWg"])))
    # second step: nothing is due any more, counters keep counting
    B.mecefo_stack_bwd_mixed(st.desc, st.attn, modes, inputs, [dict(dX=dX, **g) for g in grads], low, B.SIDE_INPUT,
                             pol, t, st.dOd, dX, 0, ws)
    torch.cuda.synchronize()
    assert list(t) == [0, 2, 0, 7]
    assert all(np.array_equal(host(P), after[1][i]) for i, P in enumerate(st.Pdev[1]))
    B.mecefo_counters_reset(t)                                          # Alg. 1: a new failure
    assert list(t) == [0, 0, 0, 0]


def test_whole_stack_pass_in_one_hip_graph():
    """Forward + chained backward of the stack captured once and replayed with fresh inputs, with
    eager work and synchronisations between the replays; every replay must equal the eager pass."""
    st = Stack(3, 2, 64, 64, 172, 4, 16, "bf16", 3)
    inputs = [I.gaussian_block_io(np.random.default_rng([36, i]), st.b, st.d, "bf16") for i in range(3)]
    eager = []
    for X, dO in inputs:
        st.X0d.copy_(dev(X, "bf16")); st.dOd.copy_(dev(dO, "bf16"))
        st.forward(); st.backward()
        eager.append(st.results())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        st.forward()
        st.backward()
    for i in (1, 2, 0, 2):
        st.X0d.copy_(dev(inputs[i][0], "bf16")); st.dOd.copy_(dev(inputs[i][1], "bf16"))
        st.dX.fill_(float("nan")); st.Xout.fill_(float("nan"))
        for g in st.grads:
            g["dWg"].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = st.results()
        assert np.array_equal(got["Xout"], eager[i]["Xout"]) and np.array_equal(got["dX"], eager[i]["dX"])
        for l in range(3):
            for k in got["grads"][l]:
                assert np.array_equal(got["grads"][l][k], eager[i]["grads"][l][k]), (i, l, k)


def test_one_training_step_two_simulated_ranks():
    """Alg. 1 for one FFN matrix on two simulated ranks: both run the degraded backward on their own
    micro-batch, Eq. (1) averages (every rank contributes to an FFN matrix), AdamW updates."""
    sts = [Stack(1, 2, 24, 32, 88, 4, 8, "f32", 4) for _ in range(2)]
    rng = np.random.default_rng(37)
    for st in sts[1:]:                      # same weights, different data
        X, dO = I.gaussian_block_io(rng, st.b, st.d, "f32")
        st.X0, st.dOut = X, dO
        st.X0d.copy_(dev(X, "f32")); st.dOd.copy_(dev(dO, "f32"))
    want_g = []
    for st in sts:
        st.forward(); st.backward()
        want_g.append(st.oracle()[2][0]["dWg"])
    n = sts[0].f * sts[0].d
    avg = torch.empty(sts[0].f, sts[0].d, device="cuda")
    B.mecefo_grad_average(B.F32, [st.grads[0]["dWg"] for st in sts], [1, 1], avg, n)
    W = sts[0].dev_layers[0]["Wg"].clone()
    M, V = torch.zeros_like(W), torch.zeros_like(W)
    B.mecefo_adamw_step(B.F32, B.F32, W, avg, M, V, n, 1, 1e-3)
    torch.cuda.synchronize()
    g = O.masked_grad_average(want_g, [1, 1])
    w, _, _ = O.adamw_step(sts[0].params[0]["Wg"], g, np.zeros_like(g), np.zeros_like(g), 1, f32(1e-3), **HP)
    assert relerr(avg.cpu().numpy(), g) < 1e-5
    assert relerr(W.cpu().numpy(), w) < 1e-6
