"""Every entry point must stay inside the workspace size its query function reports: the calls run
on a workspace of exactly that size placed in the middle of a larger buffer whose two flanks hold a
canary pattern, and the flanks must be unchanged afterwards.  Results are checked elsewhere."""
import numpy as np
import pytest
import torch

from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I

pytestmark = pytest.mark.gpu
FLANK = 1 << 20


class Guarded:
    def __init__(self, nbytes):
        self.n = nbytes
        self.buf = torch.full((nbytes + 2 * FLANK,), 0xA5, dtype=torch.uint8, device="cuda")
        self.ws = self.buf[FLANK:FLANK + nbytes]

    def check(self, what):
        torch.cuda.synchronize()
        lo, hi = self.buf[:FLANK], self.buf[FLANK + self.n:]
        assert bool((lo == 0xA5).all()) and bool((hi == 0xA5).all()), f"{what}: wrote outside its workspace"


def rnd(rows, cols, std, ld=None, dtype=torch.bfloat16):
    t = torch.zeros(rows, ld or cols, dtype=dtype, device="cuda")
    t[:, :cols] = (torch.randn(rows, cols, device="cuda") * std).to(dtype)
    return t


@pytest.mark.parametrize("batch,seq,d,f,heads,r", [(2, 300, 256, 688, 4, 64), (1, 77, 64, 200, 8, 9), (3, 520, 128, 344, 2, 32)])
def test_all_entry_points_respect_their_workspace(batch, seq, d, f, heads, r):
    torch.manual_seed(0)
    b = batch * seq
    ldf = (f + 7) // 8 * 8
    ldr = (r + 7) // 8 * 8
    desc = B.make_desc(b, d, f, B.BF16, B.F32, d, ldf, d, ldf)
    attn = B.make_attn_desc(batch, seq, heads, d)
    W = dict(Wq=rnd(d, d, d ** -0.5), Wk=rnd(d, d, d ** -0.5), Wv=rnd(d, d, d ** -0.5), Wo=rnd(d, d, d ** -0.5),
             Wg=rnd(f, d, 0.05), Wu=rnd(f, d, 0.05), Wd=rnd(d, f, 0.05, ldf),
             g_attn=torch.ones(d, dtype=torch.bfloat16, device="cuda"), g_ffn=torch.ones(d, dtype=torch.bfloat16, device="cuda"))
    X, dOut = rnd(b, d, 1.0), rnd(b, d, 1.0)
    P = [rnd(d, r, d ** -0.5, ldr), rnd(d, r, d ** -0.5, ldr), rnd(f, r, f ** -0.5, ldr)]
    projs = [B.proj(p, r) for p in P]
    act = lambda: torch.empty(b, d, dtype=torch.bfloat16, device="cuda")
    out = dict(Out=act(), H=act(), Q=act(), K=act(), V=act(), O=act(), L=torch.empty(batch * heads * seq, device="cuda"))
    g = Guarded(B.mecefo_block_fwd_workspace_bytes(desc, attn))
    B.mecefo_block_fwd(desc, attn, dict(X=X, **W), out, g.ws)
    g.check("mecefo_block_fwd")
    grads = dict(dX=act(), dg_attn=torch.zeros(d, device="cuda"), dg_ffn=torch.zeros(d, device="cuda"),
                 dWg=torch.zeros(f, d, device="cuda"), dWu=torch.zeros(f, d, device="cuda"), dWd=torch.zeros(d, ldf, device="cuda"))
    for k in ("dWq", "dWk", "dWv", "dWo"):
        grads[k] = torch.zeros(d, d, device="cuda")
    g = Guarded(B.mecefo_block_full_workspace_bytes(desc, attn))
    inp = dict(X=X, dOut=dOut, **W, **{k: out[k] for k in ("H", "Q", "K", "V", "O", "L")})
    B.mecefo_block_bwd_full(desc, attn, inp, grads, 0, g.ws)
    g.check("mecefo_block_bwd_full")
    g = Guarded(B.mecefo_workspace_bytes(desc, r, r, r))
    dgam = torch.zeros(d, device="cuda")
    for side in (B.SIDE_INPUT,):
        B.mecefo_block_bwd_skip(desc, out["H"], dOut, W["g_ffn"], W["Wg"], W["Wu"], W["Wd"], *projs, side, grads["dX"], dgam,
                                grads["dWg"], grads["dWu"], grads["dWd"], 0, g.ws)
        g.check("mecefo_block_bwd_skip")
    B.mecefo_block_bwd_skip_ex(desc, out["H"], dOut, W["g_ffn"], W["Wg"], W["Wu"], W["Wd"], *projs, B.SIDE_INPUT, grads["dX"],
                               dgam, grads["dWg"], grads["dWu"], grads["dWd"], 0, g.ws, exact_wgrad_mask=5)
    g.check("mecefo_block_bwd_skip_ex")
    B.mecefo_ffn_bwd_exact(desc, X, dOut, W["Wg"], W["Wu"], W["Wd"], None, None, grads["dX"], grads["dWg"], grads["dWu"],
                           grads["dWd"], 0, g.ws)
    g.check("mecefo_ffn_bwd_exact")
    B.mecefo_ffn_bwd_lowrank(desc, X, dOut, W["Wg"], W["Wu"], W["Wd"], *projs, B.SIDE_INPUT, grads["dX"], grads["dWg"],
                             grads["dWu"], grads["dWd"], 0, g.ws)
    g.check("mecefo_ffn_bwd_lowrank")
    g = Guarded(B.mecefo_projection_workspace_bytes(B.BF16, f, d, r))
    Pout = torch.empty_like(P[0])
    B.mecefo_projection_refresh(B.BF16, W["Wg"], f, d, d, 0, P[0], ldr, r, 2, 4, 2, Pout, ldr, g.ws)
    g.check("mecefo_projection_refresh (right)")
    g = Guarded(B.mecefo_projection_workspace_bytes(B.BF16, d, f, r, left=0))
    Pd_out = torch.empty_like(P[2])
    B.mecefo_projection_refresh(B.BF16, W["Wd"], d, f, ldf, 0, P[2], ldr, r, 2, 4, 2, Pd_out, ldr, g.ws)
    g.check("mecefo_projection_refresh (down)")
    g = Guarded(B.mecefo_stack_workspace_bytes(desc, attn, r, r, r))
    lw = B.layer_weights([W, W])
    Hs = [act(), act()]
    B.mecefo_stack_fwd_neighbor(desc, attn, lw, X, Hs, out["Out"], g.ws)
    g.check("mecefo_stack_fwd_neighbor")
    low = B.layer_lowrank([dict(Pg=projs[0], Pu=projs[1], Pd=projs[2], dg_ffn=dgam, dWg=grads["dWg"], dWu=grads["dWu"],
                                dWd=grads["dWd"]) for _ in range(2)])
    B.mecefo_stack_bwd_skip(desc, lw, Hs, low, B.SIDE_INPUT, dOut, grads["dX"], 0, g.ws)
    g.check("mecefo_stack_bwd_skip")
