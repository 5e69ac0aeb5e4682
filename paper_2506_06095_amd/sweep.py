"""Latency sweep of the masked-MHA forward over the paper's grid (Sec. 5.1 / Sec. 5.2: BERT-Base
head shape 12 x 64, fp16, sequence 128..4096, batch 1..16, the four masks of Table 2).

    python -m paper_2506_06095_amd.sweep [--seqs 128,512,...] [--batches 1,8,16] [--steps 100] [--graph]

Prints one markdown table row per (mask, batch, seq): latency of the selected kernel, of both
kernels when forced, and of PyTorch's dense scaled_dot_product_attention with the same boolean
mask (context only).  Inputs are synthetic (seeded normal Q/K/V); masks come from their pattern
descriptions, so nothing of size seq x seq is built on the host except for the dense baseline.
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def _time(fn, stream, torch, steps, warmup, graph=False):
    import time
    t_end = time.perf_counter() + 0.03  # the chip's clocks need about 30 ms of load to settle
    while time.perf_counter() < t_end:
        for _ in range(max(warmup, 1)):
            fn()
        torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if graph:
        # 20 calls captured once and replayed: the device's time per call, without the host's call rate
        per_graph = 20
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(per_graph):
                    fn()
        torch.cuda.synchronize()
        g.replay()
        replays = max(1, steps // per_graph)
        a.record(stream)
        for _ in range(replays):
            g.replay()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (replays * per_graph) * 1e3
    a.record(stream)
    for _ in range(steps):
        fn()
    b.record(stream)
    torch.cuda.synchronize()
    return a.elapsed_time(b) / steps * 1e3  # us per call, back to back


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--seqs", default="128,256,512,1024,2048,4096")
    ap.add_argument("--batches", default="1,8,16")
    ap.add_argument("--masks", default="causal,sliding_window,longformer,bigbird")
    ap.add_argument("--heads", type=int, default=12)
    ap.add_argument("--head-dim", type=int, default=64)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-dense", action="store_true", help="skip the PyTorch dense baseline")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph holding 20 calls (device time per call, no host call rate)")
    args = ap.parse_args()

    import torch
    import paper_2506_06095_amd as smha
    import workloads as W

    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    H, d = args.heads, args.head_dim
    print("| mask | batch | seq | density | selected | selected us | block us | row us | torch dense us | eff TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for name in args.masks.split(","):
        spec = W.table2_spec(name)
        for B in (int(x) for x in args.batches.split(",")):
            for S in (int(x) for x in args.seqs.split(",")):
                g = torch.Generator(device="cuda").manual_seed(S * 31 + B)
                q, k, v = (torch.randn(B, H, S, d, device="cuda", generator=g).half() for _ in range(3))
                out = torch.empty_like(q)
                us = {}
                for label, force in (("auto", smha.SMHA_KERNEL_AUTO), ("block", smha.SMHA_KERNEL_BLOCK),
                                     ("row", smha.SMHA_KERNEL_ROW)):
                    with smha.Plan.from_desc(spec, B, H, S, block=64, head_dim=d, force=force) as plan:
                        info = plan.info()
                        if label == "auto":
                            chosen = "row" if info["kernel"] == smha.SMHA_KERNEL_ROW else "block"
                            nnz = info["nnz"] * (B * H // (info["Bm"] * info["Hm"]))
                        us[label] = _time(lambda: plan.forward(q, k, v, out=out), stream, torch, args.steps, args.warmup, args.graph)
                dense_us = float("nan")
                if not args.no_dense:
                    m = torch.from_numpy(W.dense_mask(spec, B, H, S).astype(bool)).cuda()
                    dense_us = _time(lambda: torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m),
                                     stream, torch, max(20, args.steps // 4), 3, args.graph)
                    del m
                print(f"| {name} | {B} | {S} | {nnz / (B * H * S * S):.3f} | {chosen} | {us['auto']:.1f} | {us['block']:.1f} | "
                      f"{us['row']:.1f} | {dense_us:.1f} | {4.0 * nnz * d / us['auto'] / 1e6:.1f} |", flush=True)
                del q, k, v, out
    return 0


if __name__ == "__main__":
    sys.exit(main())
