"""GPU parity of the block forward (Alg. 2: the same forward in both modes; the modes differ in
what is kept) against the oracle's block_fwd_full, and the forward -> backward chains of both
modes running entirely on the library's kernels."""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O
from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I
from gpu_util import TOL, assert_close, dev, host, relerr, tdtype, poisoned_ws
from test_gpu_full_block import FullBlock, GRADS, make_case, token_major

pytestmark = pytest.mark.gpu
EPS = 1e-6


class Forward:
    def __init__(self, blk: FullBlock, heads, batch, seq):
        self.blk = blk
        b, ld = blk.b, blk.ld_d
        t = tdtype(blk.dtype)
        nan = float("nan")
        self.out = {k: torch.full((b, ld), nan, dtype=t, device="cuda") for k in ("Out", "H", "Q", "K", "V", "O")}
        self.out["L"] = torch.full((batch * heads * seq,), nan, dtype=torch.float32, device="cuda")
        self.inp = {k: blk.inp[k] for k in ("X", "g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd")}
        self.ws = poisoned_ws(B.mecefo_block_fwd_workspace_bytes(blk.desc, blk.attn))

    def run(self, neighbor=False):
        out = {k: v for k, v in self.out.items() if not neighbor or k in ("Out", "H")}
        B.mecefo_block_fwd(self.blk.desc, self.blk.attn, self.inp, out, self.ws)
        torch.cuda.synchronize()
        return {k: (host(v, self.blk.d) if v.ndim == 2 else host(v)) for k, v in out.items()}


def oracle_forward(p, X, heads, batch, seq):
    out, H, c = O.block_fwd_full(X, p, heads, batch, seq, EPS)
    b, d = X.shape
    return dict(Out=out, H=H, Q=token_major(c["Q"], b, d), K=token_major(c["K"], b, d), V=token_major(c["V"], b, d),
                O=c["O"], L=c["L"].reshape(-1))


def run_fwd(seed, batch, seq, d, f, heads, dtype, pad=0):
    p, X, dOut = make_case(seed, batch, seq, d, f, heads, dtype)
    blk = FullBlock(p, X, dOut, heads, batch, seq, dtype, pad=pad)
    fwd = Forward(blk, heads, batch, seq)
    got = fwd.run()
    want = oracle_forward(p, X, heads, batch, seq)
    errs = assert_close(got, want, TOL[dtype], label=f"fwd {dtype} B{batch} S{seq} d{d} h{heads}: ")
    return p, X, dOut, blk, fwd, got, want, errs


@pytest.mark.parametrize("batch,seq,d,f,heads", [(2, 37, 48, 100, 4), (1, 130, 64, 72, 2), (3, 9, 32, 40, 8)])
def test_block_fwd_f32_ragged(batch, seq, d, f, heads):
    print(run_fwd(21, batch, seq, d, f, heads, "f32")[-1])


@pytest.mark.parametrize("batch,seq,d,f,heads,pad", [(3, 150, 128, 344, 4, 0), (2, 77, 64, 200, 8, 8), (1, 300, 256, 512, 2, 0)])
def test_block_fwd_bf16_ragged(batch, seq, d, f, heads, pad):
    print(run_fwd(22, batch, seq, d, f, heads, "bf16", pad=pad)[-1])


@pytest.mark.parametrize("tile", ["S", "L8R", "L8"])
def test_block_fwd_bf16_forced_tiles_cross_the_diagonal(tile, mecefo_option):
    mecefo_option("tile", tile)
    print(tile, run_fwd(23, 2, 523, 256, 344, 2, "bf16")[-1])
    print(tile, run_fwd(24, 1, 768, 256, 344, 4, "bf16")[-1])


@pytest.mark.parametrize("batch,seq,d,heads,pad", [(2, 523, 256, 2, 0), (1, 768, 256, 4, 8), (3, 1, 128, 2, 0),
                                                   (2, 63, 128, 1, 0), (1, 129, 64, 1, 8), (2, 257, 512, 4, 0)])
def test_block_fwd_bf16_fused_attention_shapes(batch, seq, d, heads, pad):
    """Head dimensions 64 and 128 take the fused attention forward: single tokens, sequences shorter
    than one key block, one past a block boundary, padded row strides."""
    print(run_fwd(29, batch, seq, d, 200, heads, "bf16", pad=pad)[-1])


@pytest.mark.parametrize("batch,seq,d,heads", [(2, 523, 256, 2), (1, 768, 256, 4)])
def test_block_fwd_bf16_materialised_scores_path(batch, seq, d, heads, mecefo_option):
    """the "attention" = "gemm" switch keeps the chunked fp32-score form (the one other head dimensions use) covered
    at head dimensions 128 and 64."""
    mecefo_option("attention", "gemm")
    print(run_fwd(30, batch, seq, d, 344, heads, "bf16")[-1])


def test_fused_attention_random_shapes_forward_then_backward():
    """Seeded sweep over sequence lengths, batch sizes, head counts and both fused head dimensions: the
    forward on the GPU, then the standard-mode backward fed with the tensors that forward kept, each
    against the oracle."""
    rng = np.random.default_rng(20251017)
    for i in range(8):
        dh = int(rng.choice([64, 128]))
        heads = int(rng.integers(1, 4))
        batch = int(rng.integers(1, 4))
        seq = int(rng.integers(1, 600))
        f = int(rng.integers(1, 40)) * 8
        pad = int(rng.integers(0, 2)) * 8
        d = dh * heads
        label = f"case {i}: B{batch} S{seq} heads {heads} dh {dh} f {f} pad {pad}"
        p, X, dOut, blk, fwd, got, want, errs = run_fwd(6000 + i, batch, seq, d, f, heads, "bf16", pad=pad)
        for k in ("H", "Q", "K", "V", "O", "L"):
            blk.inp[k] = fwd.out[k]
        res = blk.run()
        ref = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)
        berrs = assert_close(res, ref, TOL["bf16"], keys=["dX"] + GRADS, label=label + " bwd: ")
        print(label, max(errs.values()), max(berrs.values()))


def test_neighbor_mode_forward_keeps_only_h_and_matches_standard_mode():
    p, X, dOut, blk, fwd, std, want, _ = run_fwd(25, 2, 200, 128, 344, 4, "bf16")
    nb = fwd.run(neighbor=True)
    assert set(nb) == {"Out", "H"}
    assert np.array_equal(nb["Out"], std["Out"]) and np.array_equal(nb["H"], std["H"])


@pytest.mark.parametrize("dtype,batch,seq,d,f,heads", [("f32", 2, 64, 64, 172, 4), ("bf16", 2, 300, 256, 688, 4)])
def test_forward_then_backward_both_modes_on_gpu(dtype, batch, seq, d, f, heads):
    """Standard mode: the saved tensors written by the GPU forward feed mecefo_block_bwd_full.
    Neighbor mode: only H is kept and feeds mecefo_block_bwd_skip.  Both against the oracle."""
    p, X, dOut, blk, fwd, got, want, _ = run_fwd(26, batch, seq, d, f, heads, dtype)
    for k in ("H", "Q", "K", "V", "O", "L"):
        blk.inp[k] = fwd.out[k]
    res = blk.run()
    ref = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)
    errs = assert_close(res, ref, TOL[dtype], keys=["dX"] + GRADS, label="fwd->full bwd: ")
    print("standard mode chain", errs)
    # neighbor mode
    from gpu_util import Layer
    r = d // 4
    rng = np.random.default_rng(5)
    Pg, Pu = I.random_orthonormal(rng, d, r, dtype), I.random_orthonormal(rng, d, r, dtype)
    Pd = I.random_orthonormal(rng, f, r, dtype)
    lay = Layer(blk.b, d, f, dtype, p["Wg"], p["Wu"], p["Wd"], p["g_ffn"], Pg, Pu, Pd, EPS)
    Hgpu = fwd.run(neighbor=True)["H"]
    res2 = lay.block_bwd_skip(Hgpu, dOut)
    ref2 = O.block_bwd_skip(want["H"], dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], Pg, Pu, Pd, EPS)
    errs2 = assert_close(res2, ref2, TOL[dtype], label="fwd->skip bwd: ")
    print("neighbor mode chain", errs2)


def test_config_c2_block_fwd():
    cfg = I.CONFIGS["C2"]
    print("C2 fwd", run_fwd(27, cfg.batch, cfg.seq, cfg.d_model, cfg.d_ff, cfg.heads, cfg.dtype)[-1])


def test_config_c5_block_fwd_whole_batch():
    """The 7B-shaped layer at its full batch (4 x 2048 tokens); the oracle walks it one sequence at a time."""
    cfg = I.CONFIGS["C5"]
    heads, batch, seq, d = cfg.heads, cfg.batch, cfg.seq, cfg.d_model
    p, X, dOut = make_case(28, batch, seq, d, cfg.d_ff, heads, cfg.dtype)
    parts = [oracle_forward(p, X[i * seq:(i + 1) * seq], heads, 1, seq) for i in range(batch)]
    want = {k: np.concatenate([q[k] for q in parts]) for k in parts[0]}
    blk = FullBlock.__new__(FullBlock)
    blk.init_from_saved(p, X, dOut, want, heads, batch, seq, cfg.dtype)
    fwd = Forward(blk, heads, batch, seq)
    got = fwd.run()
    print("C5 fwd, whole batch", assert_close(got, want, TOL["bf16"], label="C5 fwd: "))
