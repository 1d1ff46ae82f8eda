"""GPU parity of the standard-mode block backward (Alg. 3, first branch: exact gradients of the
FFN and the attention module) against the CPU oracle, through the C ABI.

The forward pass that produces the saved tensors (H, rotated Q and K, V, O and the softmax
log-sum-exp L) is the oracle's, in fp64, rounded to the storage type: the library is handed what
a forward pass on the same rank would have kept.
"""
import numpy as np
import pytest
import torch

from oracle import mecefo_oracle as O
from paper_2510_16415_amd import binding as B
from paper_2510_16415_amd import inputs as I
from gpu_util import TOL, assert_close, dev, host, tdtype, poisoned_ws

pytestmark = pytest.mark.gpu
EPS = 1e-6

GRADS = ["dg_attn", "dg_ffn", "dWq", "dWk", "dWv", "dWo", "dWg", "dWu", "dWd"]


def make_case(seed, batch, seq, d, f, heads, dtype, attn_std=None):
    rng = np.random.default_rng([20251016, seed])
    b = batch * seq
    Wg, Wu, Wd, _ = I.ffn_weights(rng, d, f, dtype, std=0.05)
    Wq, Wk, Wv, Wo, _ = I.mha_weights(rng, d, dtype, std=attn_std or 1.5 / np.sqrt(d))
    p = dict(Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, Wg=Wg, Wu=Wu, Wd=Wd,
             g_attn=I.perturbed_gain(rng, d, dtype), g_ffn=I.perturbed_gain(rng, d, dtype))
    X, dOut = I.gaussian_block_io(rng, b, d, dtype)
    return p, X, dOut


def token_major(t, b, d):
    return np.ascontiguousarray(t.transpose(0, 2, 1, 3).reshape(b, d))


class FullBlock:
    """Device buffers, descriptors and workspace for one call of mecefo_block_bwd_full."""

    def __init__(self, p, X, dOut, heads, batch, seq, dtype, grad_dtype="f32", pad=0):
        _, H, cache = O.block_fwd_full(X, p, heads, batch, seq, EPS)
        b, d = X.shape
        saved = dict(H=H, Q=token_major(cache["Q"], b, d), K=token_major(cache["K"], b, d),
                     V=token_major(cache["V"], b, d), O=cache["O"], L=cache["L"].reshape(-1))
        self.init_from_saved(p, X, dOut, saved, heads, batch, seq, dtype, grad_dtype, pad)

    def init_from_saved(self, p, X, dOut, saved, heads, batch, seq, dtype, grad_dtype="f32", pad=0):
        b, d = X.shape
        f = p["Wg"].shape[0]
        self.b, self.d, self.f, self.dtype = b, d, f, dtype
        al = 8 if dtype == "bf16" else 1
        rnd = (lambda x: (x + al - 1) // al * al)
        self.ld_d, self.ld_f = rnd(d) + pad, rnd(f) + pad
        cast = (lambda a: I.round_to_bf16_grid(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))
        self.saved = {k: cast(saved[k]) for k in ("H", "Q", "K", "V", "O")}
        act = lambda a: dev(a, dtype, self.ld_d)
        self.inp = dict(X=act(X), dOut=act(dOut), g_attn=dev(p["g_attn"], dtype), g_ffn=dev(p["g_ffn"], dtype),
                        L=torch.from_numpy(saved["L"].astype(np.float32)).cuda())
        for k, v in self.saved.items():
            self.inp[k] = act(v)
        for k in ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu"):
            self.inp[k] = dev(p[k], dtype, self.ld_d)
        self.inp["Wd"] = dev(p["Wd"], dtype, self.ld_f)
        dt = B.BF16 if dtype == "bf16" else B.F32
        gdt = B.F32 if grad_dtype == "f32" else dt
        self.desc = B.make_desc(b, d, f, dt, gdt, self.ld_d, self.ld_f, self.ld_d, self.ld_f, EPS)
        self.attn = B.make_attn_desc(batch, seq, heads, self.ld_d)
        gt = torch.float32 if grad_dtype == "f32" else tdtype(dtype)
        nan = float("nan")
        self.out = dict(dX=torch.full((b, self.ld_d), nan, dtype=tdtype(dtype), device="cuda"),
                        dg_attn=torch.full((d,), nan, dtype=gt, device="cuda"),
                        dg_ffn=torch.full((d,), nan, dtype=gt, device="cuda"),
                        dWd=torch.full((d, self.ld_f), nan, dtype=gt, device="cuda"))
        for k in ("dWq", "dWk", "dWv", "dWo"):
            self.out[k] = torch.full((d, self.ld_d), nan, dtype=gt, device="cuda")
        for k in ("dWg", "dWu"):
            self.out[k] = torch.full((f, self.ld_d), nan, dtype=gt, device="cuda")
        self.ws = poisoned_ws(B.mecefo_block_full_workspace_bytes(self.desc, self.attn))

    def run(self, accumulate=0, alias=False):
        out = dict(self.out)
        if alias:
            out["dX"] = self.inp["dOut"]
        B.mecefo_block_bwd_full(self.desc, self.attn, self.inp, out, accumulate, self.ws)
        torch.cuda.synchronize()
        res = {k: host(out[k], self.f if k == "dWd" else self.d) if out[k].ndim == 2 else host(out[k]) for k in out}
        return res


def run_case(seed, batch, seq, d, f, heads, dtype, **kw):
    p, X, dOut = make_case(seed, batch, seq, d, f, heads, dtype)
    blk = FullBlock(p, X, dOut, heads, batch, seq, dtype, **kw)
    want = O.block_bwd_full(X, dOut, p, heads, batch, seq, EPS)
    got = blk.run()
    errs = assert_close(got, want, TOL[dtype], keys=["dX"] + GRADS, label=f"{dtype} B{batch} S{seq} d{d} h{heads}: ")
    return blk, want, errs


@pytest.mark.parametrize("batch,seq,d,f,heads", [(2, 37, 48, 100, 4), (1, 130, 64, 72, 2), (3, 9, 32, 40, 8)])
def test_full_block_f32_ragged(batch, seq, d, f, heads):
    _, _, errs = run_case(1, batch, seq, d, f, heads, "f32")
    print(errs)


@pytest.mark.parametrize("batch,seq,d,f,heads", [(3, 150, 128, 344, 4), (2, 77, 64, 200, 8), (1, 300, 256, 512, 2)])
def test_full_block_bf16_ragged(batch, seq, d, f, heads):
    _, _, errs = run_case(2, batch, seq, d, f, heads, "bf16")
    print(errs)


@pytest.mark.parametrize("tile", ["S", "L4", "L8R", "L8"])
def test_full_block_bf16_forced_tiles_cross_the_diagonal(tile, mecefo_option):
    """Sequences longer than two tiles of every configuration, so that the causal clipping of the
    K loops and the skipped tiles above the diagonal are exercised; seq is not a multiple of 8."""
    mecefo_option("tile", tile)
    _, _, errs = run_case(3, 2, 523, 256, 344, 2, "bf16")
    print(tile, errs)


def test_full_block_bf16_aligned_seq_large_tiles(mecefo_option):
    """seq % 8 == 0 keeps every attention product on the direct-to-LDS kernel."""
    mecefo_option("tile", "L8")
    _, _, errs = run_case(4, 2, 768, 256, 344, 4, "bf16", pad=8)
    print(errs)


@pytest.mark.parametrize("batch,seq,d,heads", [(2, 523, 256, 2), (1, 768, 256, 4), (2, 130, 128, 2)])
def test_full_block_bf16_five_product_attention_path(batch, seq, d, heads, mecefo_option):
    """Head dimensions 64 and 128 normally take the fused dK / dV kernel; the "attention" = "gemm" switch keeps the
    five batched products (the path every other head dimension and the fp32 configuration use)."""
    mecefo_option("attention", "gemm")
    _, _, errs = run_case(9, batch, seq, d, 344, heads, "bf16")
    print(errs)


def test_full_block_accumulate_alias_and_bf16_grads():
    p, X, dOut = make_case(5, 2, 96, 128, 344, 4, "bf16")
    want = O.block_bwd_full(X, dOut, p, 4, 2, 96, EPS)
    blk = FullBlock(p, X, dOut, 4, 2, 96, "bf16", grad_dtype="bf16")
    first = blk.run()
    assert_close(first, want, TOL["bf16"], keys=["dX"] + GRADS)
    second = blk.run(accumulate=1, alias=True)    # dX written over dOut; gradients doubled
    want2 = {k: 2 * want[k] for k in GRADS}
    want2["dX"] = want["dX"]
    assert_close(second, want2, TOL["bf16"], keys=["dX"] + GRADS)


def test_full_block_rerun_is_bitwise_identical():
    p, X, dOut = make_case(6, 2, 200, 128, 344, 4, "bf16")
    blk = FullBlock(p, X, dOut, 4, 2, 200, "bf16")
    a = blk.run()
    b = blk.run()
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_full_block_empty_batch():
    d, f, heads = 64, 72, 4
    p, X, dOut = make_case(7, 1, 8, d, f, heads, "f32")
    blk = FullBlock(p, X, dOut, heads, 1, 8, "f32")
    desc = B.make_desc(0, d, f, B.F32, B.F32, d, f, d, f, EPS)
    attn = B.make_attn_desc(0, 8, heads, d)
    inp = {k: (v if k.startswith(("W", "g_")) else None) for k, v in blk.inp.items()}
    out = dict(blk.out)
    out["dX"] = None
    B.mecefo_block_bwd_full(desc, attn, inp, out, 0, blk.ws)
    torch.cuda.synchronize()
    for k in GRADS:
        assert float(out[k].abs().max()) == 0.0, k


def test_full_block_matches_skip_plus_attention_branch():
    """dX(full) - dX(skip with exact weight gradients) is the attention branch's contribution, and the
    FFN gradients of both modes coincide (Sec. 3.2: the skip changes nothing but the MHA path)."""
    p, X, dOut = make_case(8, 2, 64, 128, 344, 4, "f32")
    blk, want, _ = run_case(8, 2, 64, 128, 344, 4, "f32")
    got = blk.run()
    _, H, _ = O.block_fwd_full(X, p, 4, 2, 64, EPS)
    skip = O.block_bwd_skip_exact_wgrad(H, dOut, p["g_ffn"], p["Wg"], p["Wu"], p["Wd"], EPS)
    for k in ("dWg", "dWu", "dWd"):
        assert np.linalg.norm(got[k] - skip[k]) <= TOL["f32"] * np.linalg.norm(skip[k])
    # The branch is a difference of two gradients that are each within the fp32 tolerance of their
    # oracle values, so its own error is bounded by that tolerance times the norms that cancel.
    branch = got["dX"] - skip["dX"]
    bound = TOL["f32"] * (np.linalg.norm(got["dX"]) + np.linalg.norm(skip["dX"]))
    assert np.linalg.norm(branch - want["dX_branch"]) <= bound


def test_config_c1_full_block():
    cfg = I.CONFIGS["C1"]
    _, _, errs = run_case(11, cfg.batch, cfg.seq, cfg.d_model, cfg.d_ff, cfg.heads, cfg.dtype)
    print("C1 full block", errs)


def test_config_c2_full_block():
    cfg = I.CONFIGS["C2"]
    _, _, errs = run_case(12, cfg.batch, cfg.seq, cfg.d_model, cfg.d_ff, cfg.heads, cfg.dtype)
    print("C2 full block", errs)


def oracle_bwd_full_by_sequence(X, dOut, p, heads, batch, seq):
    """block_bwd_full of a batch as the sum over its sequences (attention never mixes sequences):
    keeps the fp64 attention tensors of one sequence in memory at a time."""
    total = None
    for i in range(batch):
        sl = slice(i * seq, (i + 1) * seq)
        g = O.block_bwd_full(X[sl], dOut[sl], p, heads, 1, seq, EPS)
        if total is None:
            total = {k: (np.zeros((batch * seq, X.shape[1])) if k in ("dX", "dH", "dX_branch") else np.zeros_like(v))
                     for k, v in g.items()}
        for k, v in g.items():
            if k in ("dX", "dH", "dX_branch"):
                total[k][sl] = v
            else:
                total[k] += v
    return total


def test_config_c5_full_block_whole_batch():
    """The 7B-shaped layer exactly as bench.py times it (4 sequences of 2048 tokens, d = 4096,
    f = 11008, 32 heads); the oracle walks the batch one sequence at a time."""
    cfg = I.CONFIGS["C5"]
    heads, batch, seq = cfg.heads, cfg.batch, cfg.seq
    p, X, dOut = make_case(15, batch, seq, cfg.d_model, cfg.d_ff, heads, cfg.dtype)
    saved = dict(H=[], Q=[], K=[], V=[], O=[], L=[])
    for i in range(batch):       # forward of the oracle, per sequence
        sl = slice(i * seq, (i + 1) * seq)
        _, H, c = O.block_fwd_full(X[sl], p, heads, 1, seq, EPS)
        saved["H"].append(H)
        for k in ("Q", "K", "V"):
            saved[k].append(token_major(c[k], seq, cfg.d_model))
        saved["O"].append(c["O"])
        saved["L"].append(c["L"].reshape(-1))
    blk = FullBlock.__new__(FullBlock)
    blk.init_from_saved(p, X, dOut, {k: np.concatenate(v) for k, v in saved.items()}, heads, batch, seq, cfg.dtype)
    want = oracle_bwd_full_by_sequence(X, dOut, p, heads, batch, seq)
    got = blk.run()
    errs = assert_close(got, want, TOL["bf16"], keys=["dX"] + GRADS, label="C5 whole batch: ")
    print("C5 full block, whole batch", errs)
