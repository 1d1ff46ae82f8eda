#!/usr/bin/env python3
"""Benchmark of the degraded (neighbor-mode) transformer-block backward on one MI355X.

A step is one pass of the whole hot path -- mecefo_block_bwd_skip: RMSNorm recompute, FFN
recompute with fused SwiGLU backward, exact Dgrad, Eq. (2) low-rank weight gradients, norm
backward + residual (the MHA skip) -- over one batch of synthetic input resident in HBM.
Workload: the LLaMA-7B-shaped layer (d=4096, f=11008, 4 x 2048 tokens, r=1024, bf16 storage,
fp32 accumulation), the configuration the headline metric is quoted on.

Prints ONE JSON line.  `value` = tokens/s through the layer, from the timed region (K steps between two
synchronisations, no per-stage events inside it).  Per-stage times, the `roofline` of the dominant kernel
stage and the shader clock come from a second pass of the same K steps with a HIP-event pair (on the
launch stream) around every stage.  `cpu_baseline` is the numpy oracle timed on the host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, vendor figure (no sparsity)
PEAK_HBM_GBS = 8000.0
PEAK_F32_VECTOR_TFLOPS = 157.3   # fp32 path of config C1: plain vector FMA

def c5_traffic_bytes():
    """HBM-side bytes per launch of the C5 GEMM stages from the two rocprofv3 --pmc runs of this script
    (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB device copy):
    the machine-readable block of profiles/gemm_bf16_C5_hbm_traffic.md, with the commit of the kernels it
    was taken on.  None when the file has no such block."""
    import re
    path = os.path.join(ROOT, "profiles", "gemm_bf16_C5_hbm_traffic.md")
    try:
        m = re.search(r"```json\s*(\{.*?\})\s*```", open(path).read(), re.S)
        return json.loads(m.group(1)) if m else None
    except OSError:
        return None


def stage_flops(b, d, f, r):
    """Algorithmic FLOPs of each GEMM stage (Sec. 3.4: 2bmn per product; Rcomp without the
    down projection, which the backward never uses)."""
    return {
        "dgrad_down": 2 * b * d * f,
        "recompute": 4 * b * d * f,
        "dgrad_gate_up": 4 * b * d * f,
        "project": 2 * b * r * (2 * d + f),
        "contract": 2 * b * r * (2 * f + d),
        "expand": 6 * r * d * f,
        "wgrad_exact": 6 * b * d * f,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C5", help="C5 (headline) or C2/C3/C4 single-layer shapes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overhead", action="store_true")
    ap.add_argument("--data", default="gaussian", choices=["gaussian", "zeros"],
                    help="zeros: every operand zero (same work, no switching in the matrix cores: shows how far "
                         "the Gaussian workload is held back by the power limit)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_16415_amd import binding as B
    from paper_2510_16415_amd import inputs as I

    if not os.path.exists(B.LIB_PATH):
        raise SystemExit(f"{B.LIB_PATH} missing: run `python -m paper_2510_16415_amd.build`")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_calibration:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = I.CONFIGS[args.config]
    b, d, f, r = cfg.tokens, cfg.d_model, cfg.d_ff, cfg.rank
    ldf = (f + 7) // 8 * 8
    gen = torch.Generator(device=dev)
    gen.manual_seed(I.BASE_SEED + cfg.index)
    bf = torch.bfloat16

    def randn(rows, cols, std=1.0, ld=None):
        t = torch.zeros(rows, ld or cols, dtype=bf, device=dev)
        if args.data == "gaussian":
            t[:, :cols] = (torch.randn(rows, cols, generator=gen, device=dev) * std).to(bf)
        return t

    # Synthetic data with the workload's distributions: weights N(0, 0.02^2), stored FFN input and
    # upstream gradient N(0, 1), gain 1; P: Gaussian columns scaled to unit norm in expectation
    # (the path treats P as opaque data, its cost does not depend on the values).
    Wg, Wu, Wd = randn(f, d, 0.02), randn(f, d, 0.02), randn(d, f, 0.02, ldf)
    H, dOut = randn(b, d), randn(b, d)
    gamma = torch.ones(d, dtype=bf, device=dev)
    Pg, Pu, Pd = randn(d, r, d ** -0.5), randn(d, r, d ** -0.5), randn(f, r, f ** -0.5)
    desc = B.make_desc(b, d, f, B.BF16, B.F32, ld_act_d=d, ld_act_f=ldf, ld_w_fd=d, ld_w_df=ldf)
    ws = torch.empty(B.mecefo_workspace_bytes(desc, r, r, r), dtype=torch.uint8, device=dev)
    dX = torch.empty_like(dOut)
    dWg = torch.zeros(f, d, dtype=torch.float32, device=dev)
    dWu = torch.zeros(f, d, dtype=torch.float32, device=dev)
    dWd = torch.zeros(d, ldf, dtype=torch.float32, device=dev)
    dgamma = torch.zeros(d, dtype=torch.float32, device=dev)
    projs = [B.proj(P, r) for P in (Pg, Pu, Pd)]

    def step():
        B.mecefo_block_bwd_skip(desc, H, dOut, gamma, Wg, Wu, Wd, *projs, B.SIDE_INPUT, dX, dgamma,
                                dWg, dWu, dWd, 0, ws)

    B.mecefo_init()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: exactly K steps between two synchronisations; one HIP-event pair around all of them.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms_per_step_events = ev0.elapsed_time(ev1) / args.steps
    # Second pass, outside the timed region: the same K steps with an event pair around every stage
    # (and the shader-clock samples of the GEMM launches).
    B.mecefo_profile_enable(16 * args.steps)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stages = B.mecefo_profile_collect()
    clocks = B.mecefo_profile_clock_mhz()
    # Third pass: per-step spread, one event pair per step on the launch stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in ev) or [ms_per_step]
    tokens_per_s = b / (ms_per_step * 1e-3)

    flops_layer = b * (10 * d * f + 6 * r * (d + f)) + 6 * r * d * f
    sf = stage_flops(b, d, f, r)
    stage_report = {}
    for name, (ms, n) in stages.items():
        avg = ms / n
        e = {"ms": round(avg, 4)}
        if name in sf:
            e["tflops"] = round(sf[name] / (avg * 1e-3) / 1e12, 1)
        if name in clocks:
            e["shader_clock_mhz"] = round(clocks[name], 0)
        stage_report[name] = e
    gemm_stages = {k: v for k, v in stage_report.items() if "tflops" in v}
    dom = max(gemm_stages, key=lambda k: gemm_stages[k]["ms"])
    dom_tflops = sf[dom] / (gemm_stages[dom]["ms"] * 1e-3) / 1e12
    # HBM-bound kernels: algorithmic bytes (bf16): norm recompute 2 b d; norm backward + residual +
    # gain-gradient partials in one pass 4 b d (dU, H, dOut in; dX out)
    hbm = {}
    if "norm_fwd" in stage_report:
        hbm["norm_fwd_GBs"] = round(2 * b * d * 2 / (stage_report["norm_fwd"]["ms"] * 1e-3) / 1e9, 1)
    if "norm_bwd" in stage_report:
        hbm["norm_bwd_GBs"] = round(4 * b * d * 2 / (stage_report["norm_bwd"]["ms"] * 1e-3) / 1e9, 1)

    # What a plain device copy of tensors of this size reaches on this machine (rotating buffers, HIP events):
    # the practical ceiling for the two norm kernels, whose tensors are 64 MiB at C5.
    nb = b * d * 2
    srcs = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(6)]
    dsts = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(6)]
    for s_, d_ in zip(srcs, dsts):
        d_.copy_(s_)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for i in range(24):
        dsts[i % 6].copy_(srcs[i % 6])
    c1.record()
    torch.cuda.synchronize()
    hbm["plain_copy_same_size_GBs"] = round(2 * nb / (c0.elapsed_time(c1) / 24 * 1e-3) / 1e9, 1)
    hbm["note"] = ("norm kernels timed inside the step (norm_fwd directly behind the previous step's 516 MB of "
                   "gradient stores); plain_copy: torch device copy of one [tokens x d_model] tensor, back to back")
    del srcs, dsts
    traffic = c5_traffic_bytes() if cfg.name == "C5" else None
    dom_clock = clocks.get(dom)
    out = {
        "metric": "degraded-block bwd tokens/sec",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: LLaMA-7B-shaped single layer, d={d} f={f} tokens={b} (4x2048) r={r}, "
                               "bf16 storage / fp32 accumulate, SIDE_INPUT projections"
                   if cfg.name == "C5" else f"{cfg.name}: one layer d={d} f={f} tokens={b} r={r}",
                   "tokens": b, "d_model": d, "d_ff": f, "rank": r},
        "ms_per_step_events": round(ms_per_step_events, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
        "ms_per_step_min": round(per_step[0], 4),
        "tflops_per_layer": round(flops_layer / (ms_per_step * 1e-3) / 1e12, 1),
        "frac_of_bf16_mfma_peak": round(flops_layer / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "algorithmic_flops_per_layer": flops_layer,
        "roofline": {"bound": "mfma", "kernel": f"gemm_bf16_dtl_kernel, launch '{dom}'",
                     "achieved": round(dom_tflops, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dom_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": (traffic or {}).get("bytes_per_launch", {}).get(dom),
                     "traffic_source": ("profiles/gemm_bf16_C5_hbm_traffic.md, kernels of commit "
                                        + str(traffic.get("commit"))) if traffic else None,
                     "flops_per_launch": sf[dom], "ms_per_launch": gemm_stages[dom]["ms"],
                     "shader_clock_mhz": round(dom_clock, 0) if dom_clock else None,
                     "peak_at_that_clock": round(PEAK_BF16_TFLOPS * dom_clock / 2400.0, 1) if dom_clock else None,
                     "timing": "HIP events on the launch stream, second pass of the same K steps"},
        "data_values": args.data,
        "stages": stage_report,
        "hbm_bound_kernels": hbm,
    }

    if not args.no_overhead:
        out["overhead_vs_full_bwd"] = overhead(B, torch, desc, b, d, f, r, ldf, H, dOut, Wg, Wu, Wd, projs, dX,
                                              dWg, dWu, dWd, ws, ms_per_step, cfg)
    if not args.no_overhead:
        out["projection_refresh"] = projection_refresh(B, torch, Wg, Wd, Pg, Pd, d, f, ldf, r, ms_per_step)
    if not args.no_overhead:
        out["variants"] = variants(B, torch, desc, b, d, f, r, ldf, H, dOut, gamma, Wg, Wu, Wd, (Pg, Pu, Pd), dX,
                                   dgamma, dWg, dWu, dWd)
        out["neighbor_stack"] = neighbor_stack(B, torch, I)
        out["step_compositions_per_layer"] = step_compositions(B, torch, I)
        out["per_config_one_layer"] = per_config_lines(B, torch, I)
        out["vendor_gemm_reference"] = vendor_gemm_reference(torch, b, d, f, args.data)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


def overhead(B, torch, desc, b, d, f, r, ldf, U, dY, Wg, Wu, Wd, projs, dU, dWg, dWu, dWd, ws, deg_block_ms, cfg):
    """Normal-vs-degraded step time, all with this library's kernels.  (A) FFN only: Eq. (2) backward
    vs the exact backward from saved activations (12bdf) vs recompute + exact Wgrad (16bdf).
    (B) whole block: mecefo_block_bwd_full (exact FFN + attention backward from the tensors a forward
    pass keeps; they are fabricated with torch outside the timed region) vs the degraded block."""
    dev = U.device
    bf = torch.bfloat16
    G = torch.empty(b, ldf, dtype=bf, device=dev)
    Z = torch.empty_like(G)
    A = torch.empty_like(G)
    B.mecefo_ffn_fwd_recompute(desc, U, Wg, Wu, None, G, Z, A, None, ws)

    def timed(fn, n=5):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    t_lr = timed(lambda: B.mecefo_ffn_bwd_lowrank(desc, U, dY, Wg, Wu, Wd, *projs, B.SIDE_INPUT, dU, dWg, dWu,
                                                  dWd, 0, ws))
    t_saved = timed(lambda: B.mecefo_ffn_bwd_exact(desc, U, dY, Wg, Wu, Wd, G, Z, dU, dWg, dWu, dWd, 0, ws))
    t_rec = timed(lambda: B.mecefo_ffn_bwd_exact(desc, U, dY, Wg, Wu, Wd, None, None, dU, dWg, dWu, dWd, 0, ws))
    del G, Z, A

    # whole block, standard mode
    heads, S, nb = cfg.heads, cfg.seq, cfg.batch
    dh = d // heads
    gen = torch.Generator(device=dev)
    gen.manual_seed(12345 + cfg.index)
    rn = lambda rows, cols, std=1.0: (torch.randn(rows, cols, generator=gen, device=dev) * std).to(bf)
    inp = dict(X=rn(b, d), H=U, dOut=dY, g_attn=torch.ones(d, dtype=bf, device=dev),
               g_ffn=torch.ones(d, dtype=bf, device=dev), Wg=Wg, Wu=Wu, Wd=Wd,
               Q=rn(b, d), K=rn(b, d), V=rn(b, d), O=rn(b, d, 0.1))
    for k in ("Wq", "Wk", "Wv", "Wo"):
        inp[k] = rn(d, d, 0.02)
    L = torch.empty(nb, heads, S, dtype=torch.float32, device=dev)
    mask = torch.triu(torch.ones(S, S, dtype=torch.bool, device=dev), 1)
    for i in range(nb):      # log-sum-exp of the causal scaled scores of the fabricated Q, K
        q = inp["Q"][i * S:(i + 1) * S].view(S, heads, dh).transpose(0, 1).float()
        k = inp["K"][i * S:(i + 1) * S].view(S, heads, dh).transpose(0, 1).float()
        sc = (q @ k.transpose(1, 2)) / dh ** 0.5
        L[i] = torch.logsumexp(sc.masked_fill(mask, float("-inf")), dim=-1)
        del q, k, sc
    inp["L"] = L.reshape(-1)
    attn = B.make_attn_desc(nb, S, heads, d)
    wsf = torch.empty(B.mecefo_block_full_workspace_bytes(desc, attn), dtype=torch.uint8, device=dev)
    grads = dict(dX=torch.empty(b, d, dtype=bf, device=dev), dg_attn=torch.zeros(d, device=dev),
                 dg_ffn=torch.zeros(d, device=dev), dWg=dWg, dWu=dWu, dWd=dWd)
    for k in ("dWq", "dWk", "dWv", "dWo"):
        grads[k] = torch.zeros(d, d, device=dev)
    full = lambda: B.mecefo_block_bwd_full(desc, attn, inp, grads, 0, wsf)
    t_full = timed(full, 10)
    # forward of the block in both modes (standard keeps Q, K, V, O, L, H; neighbor keeps H)
    wsw = torch.empty(B.mecefo_block_fwd_workspace_bytes(desc, attn), dtype=torch.uint8, device=dev)
    fin = {k: inp[k] for k in ("X", "g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd")}
    act = lambda: torch.empty(b, d, dtype=bf, device=dev)
    fout = dict(Out=act(), H=act(), Q=act(), K=act(), V=act(), O=act(), L=torch.empty(nb * heads * S, device=dev))
    t_fwd_std = timed(lambda: B.mecefo_block_fwd(desc, attn, fin, fout, wsw), 5)
    t_fwd_nb = timed(lambda: B.mecefo_block_fwd(desc, attn, fin, dict(Out=fout["Out"], H=fout["H"]), wsw), 5)
    del wsw, fout
    B.mecefo_profile_enable(32 * 5)
    for _ in range(5):
        full()
    torch.cuda.synchronize()
    stages = {k: round(ms / 5, 4) for k, (ms, n) in B.mecefo_profile_collect().items()}
    # attention core FLOPs with the causal half: five [S x S x dh] products per (sequence, head)
    core_flops = 5 * nb * heads * S * S * dh
    core_ms = sum(stages.get(k, 0.0) for k in ("attn_probs", "attn_dv", "attn_ds", "attn_dq", "attn_dk", "attn_fused_kv"))
    full_flops = 16 * b * d * f + 16 * b * d * d + core_flops
    # Bound on how much the comparator's slower attention core flatters the ratio: the full block's time if
    # its attention core ran at the rate the rest of that block reaches (its GEMM launches).
    rest_rate = (full_flops - core_flops) / max(t_full - core_ms, 1e-9)
    t_full_fast_core = t_full - core_ms + core_flops / rest_rate
    return {
        "ffn_degraded_lowrank_ms": round(t_lr, 4),
        "ffn_exact_from_saved_ms": round(t_saved, 4),
        "ffn_recompute_exact_wgrad_ms": round(t_rec, 4),
        "ffn_degraded_over_exact": round(t_lr / t_saved, 4),
        "block_degraded_ms": round(deg_block_ms, 4),
        "block_full_ms": round(t_full, 4),
        "block_degraded_over_full": round(deg_block_ms / t_full, 4),
        "block_degraded_over_full_if_attention_core_ran_at_the_rate_of_the_rest": round(deg_block_ms / t_full_fast_core, 4),
        "block_full_tflops": round(full_flops / (t_full * 1e-3) / 1e12, 1),
        "block_fwd_standard_ms": round(t_fwd_std, 4),
        "block_fwd_neighbor_ms": round(t_fwd_nb, 4),
        "attention_core_ms": round(core_ms, 4),
        "attention_core_tflops": round(core_flops / (core_ms * 1e-3) / 1e12, 1) if core_ms > 0 else None,
        "block_full_stages_ms": stages,
        "note": "block_full: FFN recomputed from H with exact weight gradients + attention backward from "
                "saved Q, K, V, O, L (fabricated outside the timed region); all kernels are this library's",
    }


def vendor_gemm_reference(torch, b, d, f, data):
    """Context, not a target and not on the product path: the vendor GEMM library (torch.matmul on bf16
    tensors) on the three large products of the step, same shapes, same kind of operands, same box and
    minute.  The matrix cores are power-limited on Gaussian operands (the shader clock drops well below
    2.4 GHz), so what any kernel can reach on this workload is best read next to this line."""
    dev, bf = torch.device("cuda:0"), torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(7)

    def mk(rows, cols, std):
        if data == "zeros":
            return torch.zeros(rows, cols, dtype=bf, device=dev)
        return (torch.randn(rows, cols, generator=g, device=dev) * std).to(bf)

    U, dOut, dGZ = mk(b, d, 1.0), mk(b, d, 1.0), mk(b, 2 * f, 1.0)
    Wgu, Wd = mk(2 * f, d, 0.02), mk(d, f, 0.02)
    cases = {
        "recompute_shape_b_x_2f_x_d_NT": (lambda: torch.matmul(U, Wgu.t()), 4 * b * d * f),
        "dgrad_down_shape_b_x_f_x_d_NN": (lambda: torch.matmul(dOut, Wd), 2 * b * d * f),
        "dgrad_gate_up_shape_b_x_d_x_2f_NN": (lambda: torch.matmul(dGZ, Wgu), 4 * b * d * f),
    }
    out = {}
    for name, (fn, fl) in cases.items():
        for _ in range(5):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(fl / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e12, 1)
    out["unit"] = "TFLOP/s"
    out["note"] = ("torch.matmul (vendor library) on plain products of the same shapes; no fused SwiGLU "
                   "backward, no second K segment: a context figure for the power-limited ceiling")
    return out


def projection_refresh(B, torch, Wg, Wd, Pg, Pd, d, f, ldf, r, deg_block_ms, tau=100):
    """Alg. 3's projection refresh (every tau = 100 neighbor steps in the paper's runs) with the
    library's SVD-free subspace iteration: one gate/up-shaped matrix ([f x d], basis in R^d) and the
    down projection ([d x f], basis in R^f); cold start = 8 rounds from Gaussian noise, warm start =
    2 rounds from the previous projection; 8 conditioning steps per round, 3 polishing steps.  Amortised cost per step = (2 gate/up + 1 down) / tau."""
    dev = Wg.device

    def timed(fn, n=3):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    res = {}
    for name, W, m, n, ldw, P in (("gate_up", Wg, f, d, d, Pg), ("down", Wd, d, f, ldf, Pd)):
        ws = torch.empty(B.mecefo_projection_workspace_bytes(B.BF16, m, n, r), dtype=torch.uint8, device=dev)
        out = torch.empty_like(P)
        for label, rounds in (("cold_8_rounds", 8), ("warm_2_rounds", 2)):
            res[f"{name}_{label}_ms"] = round(timed(lambda: B.mecefo_projection_refresh(
                B.BF16, W, m, n, ldw, 0, P, P.stride(0), r, rounds, 8, 3, out, out.stride(0), ws)), 3)
        del ws
    per_step = (2 * res["gate_up_warm_2_rounds_ms"] + res["down_warm_2_rounds_ms"]) / tau
    res["amortised_ms_per_step_tau100_warm"] = round(per_step, 4)
    res["amortised_fraction_of_degraded_block"] = round(per_step / deg_block_ms, 4)
    return res


def variants(B, torch, desc, b, d, f, r, ldf, H, dOut, gamma, Wg, Wu, Wd, Ps, dX, dgamma, dWg, dWu, dWd):
    """The knobs the paper names (extra checkpoints, no low-rank approximation, other ranks), timed with
    mecefo_block_bwd_skip_ex on the same layer; ms per call."""
    dev = H.device
    bf = torch.bfloat16

    def timed(fn, n=10):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    res = {}
    G = torch.empty(b, ldf, dtype=bf, device=dev)
    Z = torch.empty_like(G)
    A = torch.empty_like(G)
    U = torch.empty_like(H)
    ws0 = torch.empty(B.mecefo_workspace_bytes(desc, r, r, r), dtype=torch.uint8, device=dev)
    B.mecefo_ffn_fwd_recompute(desc, H, Wg, Wu, None, G, Z, A, None, ws0)     # values only need to be finite
    del A, U

    def call(ranks, ws, **kw):
        Pr = [B.proj(P, rk) if rk else None for P, rk in zip(Ps, ranks)]
        return lambda: B.mecefo_block_bwd_skip_ex(desc, H, dOut, gamma, Wg, Wu, Wd, *Pr, B.SIDE_INPUT, dX, dgamma,
                                                  dWg, dWu, dWd, 0, ws, **kw)

    res["default_r%d_ms" % r] = round(timed(call((r, r, r), ws0)), 4)
    res["saved_G_Z_r%d_ms" % r] = round(timed(call((r, r, r), ws0, G=G, Z=Z)), 4)
    res["exact_wgrad_all_ms"] = round(timed(call((0, 0, 0), ws0, exact_wgrad_mask=7)), 4)
    for rk in (r // 4, r // 2):
        res["default_r%d_ms" % rk] = round(timed(call((rk, rk, rk), ws0)), 4)
    return res


def neighbor_stack(B, torch, I, name="C2"):
    """A whole neighbor-mode pass over the layers of a small stack config (launch-bound): forward keeping
    only H_l, then the chained degraded backward, eager and replayed from one HIP graph; plus the
    activation bytes each mode keeps per layer."""
    cfg = I.CONFIGS[name]
    dev = torch.device("cuda:0")
    b, d, f, r, L = cfg.tokens, cfg.d_model, cfg.d_ff, cfg.rank, cfg.layers
    ldf = (f + 7) // 8 * 8
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(777 + cfg.index)

    def rn(rows, cols, std=1.0, ld=None):
        t = torch.zeros(rows, ld or cols, dtype=bf, device=dev)
        t[:, :cols] = (torch.randn(rows, cols, generator=gen, device=dev) * std).to(bf)
        return t

    desc = B.make_desc(b, d, f, B.BF16, B.F32, d, ldf, d, ldf)
    attn = B.make_attn_desc(cfg.batch, cfg.seq, cfg.heads, d)
    layers, low, keep = [], [], []
    for _ in range(L):
        e = dict(g_attn=torch.ones(d, dtype=bf, device=dev), g_ffn=torch.ones(d, dtype=bf, device=dev),
                 Wq=rn(d, d, d ** -0.5), Wk=rn(d, d, d ** -0.5), Wv=rn(d, d, d ** -0.5), Wo=rn(d, d, d ** -0.5),
                 Wg=rn(f, d, 0.02), Wu=rn(f, d, 0.02), Wd=rn(d, f, 0.02, ldf))
        P = [rn(d, r, d ** -0.5), rn(d, r, d ** -0.5), rn(f, r, f ** -0.5)]
        g = dict(dg_ffn=torch.zeros(d, device=dev), dWg=torch.zeros(f, d, device=dev),
                 dWu=torch.zeros(f, d, device=dev), dWd=torch.zeros(d, ldf, device=dev))
        keep.append((e, P, g))
        layers.append(e)
        low.append(dict(Pg=B.proj(P[0], r), Pu=B.proj(P[1], r), Pd=B.proj(P[2], r), **g))
    lw, lr = B.layer_weights(layers), B.layer_lowrank(low)
    H = [torch.empty(b, d, dtype=bf, device=dev) for _ in range(L)]
    X0, dOut = rn(b, d), rn(b, d)
    Xout, dX = torch.empty_like(X0), torch.empty_like(X0)
    ws = torch.empty(B.mecefo_stack_workspace_bytes(desc, attn, r, r, r), dtype=torch.uint8, device=dev)

    def fwd():
        B.mecefo_stack_fwd_neighbor(desc, attn, lw, X0, H, Xout, ws)

    def bwd():
        B.mecefo_stack_bwd_skip(desc, lw, H, lr, B.SIDE_INPUT, dOut, dX, 0, ws)

    def timed(fn, n=20):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    t_fwd, t_bwd = timed(fwd), timed(bwd)
    graphs = []
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for fn in (fwd, bwd):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
        graphs.append(g)
    torch.cuda.current_stream().wait_stream(side)
    g_fwd, g_bwd = timed(graphs[0].replay), timed(graphs[1].replay)
    dh = d // cfg.heads
    kept_neighbor = b * d * 2
    kept_standard = 5 * b * d * 2 + cfg.batch * cfg.heads * cfg.seq * 4
    return {
        "config": f"{name}: {L} layers, tokens={b}, d={d}, f={f}, heads={cfg.heads}, r={r}, bf16",
        "fwd_eager_ms": round(t_fwd, 4), "fwd_graph_ms": round(g_fwd, 4),
        "bwd_skip_eager_ms": round(t_bwd, 4), "bwd_skip_graph_ms": round(g_bwd, 4),
        "bwd_tokens_per_s_graph": round(b / (g_bwd * 1e-3), 1),
        "activation_bytes_kept_per_layer": {
            "neighbor_mode_H_only": kept_neighbor,
            "standard_mode_H_Q_K_V_O_L": kept_standard,
            "standard_mode_with_saved_G_Z": kept_standard + 2 * b * ldf * 2,
        },
    }


def step_compositions(B, torch, I, names=("C3", "C4")):
    """Per-layer backward time of one node's step in the three compositions the method implies:
    healthy (one standard-mode backward), neighbor as in Alg. 3 (own and absorbed micro-batch both in
    neighbor mode; the second accumulates), and neighbor with only the absorbed micro-batch degraded
    (standard-mode backward of the own one + a degraded one accumulating into the same buffers)."""
    dev = torch.device("cuda:0")
    bf = torch.bfloat16
    out = {}
    for name in names:
        cfg = I.CONFIGS[name]
        b, d, f, r = cfg.tokens, cfg.d_model, cfg.d_ff, cfg.rank
        ldf = (f + 7) // 8 * 8
        gen = torch.Generator(device=dev)
        gen.manual_seed(4242 + cfg.index)

        def rn(rows, cols, std=1.0, ld=None):
            t = torch.zeros(rows, ld or cols, dtype=bf, device=dev)
            t[:, :cols] = (torch.randn(rows, cols, generator=gen, device=dev) * std).to(bf)
            return t

        desc = B.make_desc(b, d, f, B.BF16, B.F32, d, ldf, d, ldf)
        attn = B.make_attn_desc(cfg.batch, cfg.seq, cfg.heads, d)
        ones = lambda: torch.ones(d, dtype=bf, device=dev)
        inp = dict(X=rn(b, d), H=rn(b, d), dOut=rn(b, d), g_attn=ones(), g_ffn=ones(),
                   Wg=rn(f, d, 0.02), Wu=rn(f, d, 0.02), Wd=rn(d, f, 0.02, ldf),
                   Q=rn(b, d), K=rn(b, d), V=rn(b, d), O=rn(b, d, 0.1))
        for k in ("Wq", "Wk", "Wv", "Wo"):
            inp[k] = rn(d, d, 0.02)
        # timing only: a constant log-sum-exp keeps every probability finite and below one
        inp["L"] = torch.full((cfg.batch * cfg.heads * cfg.seq,), 30.0, device=dev)
        Ps = [rn(d, r, d ** -0.5), rn(d, r, d ** -0.5), rn(f, r, f ** -0.5)]
        projs = [B.proj(P, r) for P in Ps]
        grads = dict(dX=torch.empty(b, d, dtype=bf, device=dev), dg_attn=torch.zeros(d, device=dev),
                     dg_ffn=torch.zeros(d, device=dev), dWg=torch.zeros(f, d, device=dev),
                     dWu=torch.zeros(f, d, device=dev), dWd=torch.zeros(d, ldf, device=dev))
        for k in ("dWq", "dWk", "dWv", "dWo"):
            grads[k] = torch.zeros(d, d, device=dev)
        ws = torch.empty(max(B.mecefo_block_full_workspace_bytes(desc, attn), B.mecefo_workspace_bytes(desc, r, r, r)),
                         dtype=torch.uint8, device=dev)

        def full(acc):
            B.mecefo_block_bwd_full(desc, attn, inp, grads, acc, ws)

        def skip(acc):
            B.mecefo_block_bwd_skip(desc, inp["H"], inp["dOut"], inp["g_ffn"], inp["Wg"], inp["Wu"], inp["Wd"], *projs,
                                    B.SIDE_INPUT, grads["dX"], grads["dg_ffn"], grads["dWg"], grads["dWu"], grads["dWd"],
                                    acc, ws)

        def timed(fn, n=20):
            fn()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) * 1e3 / n

        t_h = timed(lambda: full(0))
        t_n = timed(lambda: (skip(0), skip(1)))
        t_m = timed(lambda: (full(0), skip(1)))
        out[name] = {
            "layer": f"tokens={b} per micro-batch, d={d}, f={f}, heads={cfg.heads}, seq={cfg.seq}, r={r}",
            "healthy_one_standard_bwd_ms": round(t_h, 4),
            "neighbor_two_degraded_bwd_ms": round(t_n, 4),
            "neighbor_standard_plus_degraded_bwd_ms": round(t_m, 4),
            "neighbor_over_healthy": round(t_n / t_h, 3),
        }
    return out


def cpu_baseline(cfg):
    """The numpy oracle, as it stands, timed on the host cores on the same layer.  `value` is its fp64 form
    (the one the parity tests compare against) over whole passes of the batch; `legs` adds its float32 form
    (numpy BLAS sgemm) on all cores over the whole batch and on one thread over a bounded token sample."""
    import numpy as np

    from oracle import mecefo_oracle as O
    from paper_2510_16415_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        threads = os.cpu_count()
    bs = cfg.tokens
    d, f, r = cfg.d_model, cfg.d_ff, cfg.rank
    rng = I.rng_for(cfg.index, 7)
    Wg, Wu, Wd, gamma = I.ffn_weights(rng, d, f, cfg.dtype)
    H, dOut = I.gaussian_block_io(rng, bs, d, cfg.dtype)
    Ps = [I._normal(rng, (n, r), n ** -0.5) for n in (d, d, f)]

    def run(tokens, dtype, budget_s, max_passes):
        t = time.perf_counter()
        passes = 0
        while True:
            O.block_bwd_skip(H[:tokens], dOut[:tokens], gamma, Wg, Wu, Wd, *Ps, 1e-6, dtype=dtype)
            passes += 1
            dt = time.perf_counter() - t
            if dt >= budget_s or passes >= max_passes:
                return passes, dt

    passes, dt = run(bs, np.float64, 8.0, 6)
    out = {"value": round(passes * bs / dt, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": f"{passes} passes over the {bs} tokens of the same layer, fp64 numpy, {dt:.1f} s"}
    legs = {}
    p32, dt32 = run(bs, np.float32, 5.0, 6)
    legs["fp32_all_cores"] = {"value": round(p32 * bs / dt32, 1), "unit": "tokens/s", "cores": int(threads),
                              "sample": f"{p32} passes over {bs} tokens, float32 numpy, {dt32:.1f} s"}
    if threadpool_limits is not None:
        sample = max(1, min(bs, 512))
        with threadpool_limits(limits=1):
            p1, dt1 = run(sample, np.float32, 6.0, 2)
        legs["fp32_one_thread"] = {"value": round(p1 * sample / dt1, 1), "unit": "tokens/s", "cores": 1,
                                   "sample": f"{p1} pass(es) over the first {sample} tokens (the token-independent "
                                             f"expand products of Eq. (2) included once per pass), float32 numpy, {dt1:.1f} s"}
    # The smaller configs' layer shapes, float32 numpy: all cores (best of three passes) and one thread.
    small = {}
    for name in ("C1", "C2", "C3", "C4"):
        c = I.CONFIGS[name]
        rg = I.rng_for(c.index, 7)
        w = I.ffn_weights(rg, c.d_model, c.d_ff, c.dtype)
        h, do = I.gaussian_block_io(rg, c.tokens, c.d_model, c.dtype)
        ps = [I._normal(rg, (n, c.rank), n ** -0.5) for n in (c.d_model, c.d_model, c.d_ff)]

        def best(n=3):
            ts = []
            for _ in range(n):
                t = time.perf_counter()
                O.block_bwd_skip(h, do, w[3], w[0], w[1], w[2], *ps, 1e-6, dtype=np.float32)
                ts.append(time.perf_counter() - t)
            return min(ts)

        e = {"tokens": c.tokens, "all_cores_tokens_per_s": round(c.tokens / best(), 1)}
        if threadpool_limits is not None:
            with threadpool_limits(limits=1):
                e["one_thread_tokens_per_s"] = round(c.tokens / best(1 if name in ("C3", "C4") else 3), 1)
        small[name] = e
    legs["fp32_one_layer_small_configs"] = small
    # Pure-loop form (explicit index sums, no numpy) on the tiny config C1's layer shape, a few tokens.
    from oracle import mecefo_loops as LO
    c1 = I.CONFIGS["C1"]
    rng1 = I.rng_for(c1.index, 7)
    W1 = I.ffn_weights(rng1, c1.d_model, c1.d_ff, c1.dtype)
    tok = 4
    H1, dO1 = I.gaussian_block_io(rng1, tok, c1.d_model, c1.dtype)
    P1 = [I._normal(rng1, (n, c1.rank), n ** -0.5) for n in (c1.d_model, c1.d_model, c1.d_ff)]
    args = [x.tolist() for x in (H1, dO1, W1[3], W1[0], W1[1], W1[2], *P1)]
    t = time.perf_counter()
    LO.block_bwd_skip_loops(*args, 1e-6)
    dtl = time.perf_counter() - t
    legs["pure_loops_C1_shape"] = {"value": round(tok / dtl, 2), "unit": "tokens/s", "cores": 1,
                                   "sample": f"one pass over {tok} tokens of the C1 layer (d={c1.d_model}, f={c1.d_ff}, "
                                             f"r={c1.rank}; the token-independent expand products dominate), pure Python loops, {dtl:.1f} s"}
    out["legs"] = legs
    return out


def per_config_lines(B, torch, I, names=("C1", "C2", "C3", "C4")):
    """Degraded-block backward of ONE layer of each smaller config (parity configs, launch- and
    occupancy-bound): tokens/s, algorithmic TFLOP/s and fraction of the peak of the arithmetic type."""
    dev = torch.device("cuda:0")
    out = {}
    for name in names:
        cfg = I.CONFIGS[name]
        b, d, f, r = cfg.tokens, cfg.d_model, cfg.d_ff, cfg.rank
        bf16 = cfg.dtype == "bf16"
        t = torch.bfloat16 if bf16 else torch.float32
        ldf = (f + 7) // 8 * 8 if bf16 else f
        gen = torch.Generator(device=dev)
        gen.manual_seed(999 + cfg.index)

        def rn(rows, cols, std=1.0, ld=None):
            x = torch.zeros(rows, ld or cols, dtype=t, device=dev)
            x[:, :cols] = (torch.randn(rows, cols, generator=gen, device=dev) * std).to(t)
            return x

        desc = B.make_desc(b, d, f, B.BF16 if bf16 else B.F32, B.F32, d, ldf, d, ldf)
        Wg, Wu, Wd = rn(f, d, 0.02), rn(f, d, 0.02), rn(d, f, 0.02, ldf)
        H, dOut = rn(b, d), rn(b, d)
        gamma = torch.ones(d, dtype=t, device=dev)
        rr = (r + 7) // 8 * 8 if bf16 else r
        Ps = [rn(d, r, d ** -0.5, rr), rn(d, r, d ** -0.5, rr), rn(f, r, f ** -0.5, rr)]
        projs = [B.proj(P, r) for P in Ps]
        ws = torch.empty(B.mecefo_workspace_bytes(desc, r, r, r), dtype=torch.uint8, device=dev)
        dX = torch.empty_like(dOut)
        g = [torch.zeros(f, d, device=dev), torch.zeros(f, d, device=dev), torch.zeros(d, ldf, device=dev),
             torch.zeros(d, device=dev)]

        def step():
            B.mecefo_block_bwd_skip(desc, H, dOut, gamma, Wg, Wu, Wd, *projs, B.SIDE_INPUT, dX, g[3], g[0], g[1],
                                    g[2], 0, ws)

        for _ in range(10):
            step()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
        for e0, e1 in ev:
            e0.record()
            step()
            e1.record()
        torch.cuda.synchronize()
        ts = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
        ms = ts[len(ts) // 2]
        flops = b * (10 * d * f + 6 * r * (d + f)) + 6 * r * d * f
        peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_VECTOR_TFLOPS
        out[name] = {"layer": f"tokens={b}, d={d}, f={f}, r={r}, {cfg.dtype}" + (" (plain FMA path, untuned)" if not bf16 else ""),
                     "ms_per_layer_median": round(ms, 4), "ms_per_layer_min": round(ts[0], 4),
                     "tokens_per_s": round(b / (ms * 1e-3), 1),
                     "tflops_per_layer": round(flops / (ms * 1e-3) / 1e12, 2),
                     "frac_of_peak": round(flops / (ms * 1e-3) / 1e12 / peak, 4),
                     "peak_tflops": peak}
    return out


if __name__ == "__main__":
    main()
