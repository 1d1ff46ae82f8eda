"""Child process of test_gpu_graph_init.py: in a fresh process, mecefo_init() and then the very first
library call on the device is made under HIP-graph capture.  Prints OK when the replays equal an
eager call made afterwards, bit for bit."""
import os
import sys

import torch

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), ".."))
from paper_2510_16415_amd import binding as B  # noqa: E402


def main():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.mecefo_init()
    B.mecefo_set_option("tile", sys.argv[1] if len(sys.argv) > 1 else "auto")
    b, d, f, r = 768, 512, 1032, 128
    bf = torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    rn = lambda rows, cols, std=1.0: (torch.randn(rows, cols, generator=g, device=dev) * std).to(bf)
    H, dOut = rn(b, d), rn(b, d)
    gamma = (1 + 0.1 * torch.randn(d, generator=g, device=dev)).to(bf)
    Wg, Wu, Wd = rn(f, d, 0.05), rn(f, d, 0.05), rn(d, f, 0.05)
    Pt = [rn(n, r, n ** -0.5) for n in (d, d, f)]
    P = [B.proj(t, r) for t in Pt]
    desc = B.make_desc(b, d, f, B.BF16)
    ws = torch.empty(B.mecefo_workspace_bytes(desc, r, r, r), dtype=torch.uint8, device=dev)

    def outputs():
        return dict(dX=torch.full((b, d), float("nan"), dtype=bf, device=dev), dgamma=torch.zeros(d, device=dev),
                    dWg=torch.zeros(f, d, device=dev), dWu=torch.zeros(f, d, device=dev),
                    dWd=torch.zeros(d, f, device=dev))

    def call(o):
        B.mecefo_block_bwd_skip(desc, H, dOut, gamma, Wg, Wu, Wd, *P, B.SIDE_INPUT, o["dX"], o["dgamma"],
                                o["dWg"], o["dWu"], o["dWd"], 0, ws)

    og = outputs()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):      # first library call of this process on the device
        call(og)
    print("captured", flush=True)
    results = []
    for _ in range(3):
        for t in og.values():
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        results.append({k: v.clone() for k, v in og.items()})
    oe = outputs()
    call(oe)
    torch.cuda.synchronize()
    for i, res in enumerate(results):
        for k in oe:
            assert torch.isfinite(res[k].float()).all(), f"replay {i}: {k} not finite"
            assert torch.equal(res[k], oe[k]), f"replay {i}: {k} differs from the eager call"
    print("OK", flush=True)


if __name__ == "__main__":
    main()
