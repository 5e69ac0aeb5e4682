#!/usr/bin/env python3
"""Benchmark of the masked-MHA hot path on one MI355X.

One step = one smha_forward launch (the fused masked-attention kernel, plus the small merge
kernel when query tiles were split) over one batch of synthetic Q/K/V resident in HBM.  The mask
is analysed once, before the timed region (the paper analyses a mask once per model, Sec. 4.2.1 /
Sec. 5.6); its cost is reported separately as `plan_ms`.

Prints ONE JSON line.  metric: effective TFLOP/s over unmasked entries (4*nnz*d*B*H flops per
step) with ms_per_step the latency; roofline: unmasked-tile flops per launch against the MI355X
dense fp16 MFMA peak; cpu_baseline: the fp64 oracle on a sample of heads of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0}   # MI355X dense MFMA, published
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel: constants copied from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# summaries under profiles/ (runs of this very command, scaled by what the same counters read for a 256 MiB device
# copy: FETCH_SIZE x2.0, WRITE_SIZE x1.0 on this machine).  This run does not measure them; the line says so.
MEASURED_TRAFFIC = {  # (workload, kernel as smha_kernel_name gives it)
    ("cfg5_bigbird_8k", "smha_block_fwd16"): {"read_bytes": 329.2e6, "write_bytes": 82.8e6},
    ("cfg5_bigbird_8k", "smha_block_fwd"): {"read_bytes": 310.2e6, "write_bytes": 82.3e6},
    ("cfg4_random_blocks", "smha_block_fwd"): {"read_bytes": 50.8e6, "write_bytes": 16.8e6},
    ("cfg3_strided_causal", "smha_row_fwd"): {"read_bytes": 59.1e6, "write_bytes": 16.8e6},
    ("cfg3_strided_causal", "smha_block_fwd"): {"read_bytes": 58.2e6, "write_bytes": 19.9e6},
    ("scattered_2048_k8", "smha_row_fwd"): {"read_bytes": 51.1e6, "write_bytes": 16.8e6},
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (5 = BigBird, seq 8192)")
    ap.add_argument("--kernel", choices=["auto", "row", "block"], default="auto")
    ap.add_argument("--block-form", type=int, default=0, choices=[0, 1, 2, 3],
                    help="which form of the block kernel runs where several exist (0 = the library's choice)")
    ap.add_argument("--scattered", type=int, default=0, metavar="K",
                    help="instead of --config: a scattered mask (K pseudo-random keys per query plus the diagonal), batch 4, "
                         "16 heads, sequence 2048, head size 64, fp16 -- the ground on which the selector takes the "
                         "row-wise kernel (not one of the five configurations; for its roofline line and profile)")
    ap.add_argument("--prewarm-ms", type=float, default=80.0,
                    help="untimed forwards for this long before the W warm-up steps: the chip's clocks take "
                         "about 30 ms of load to settle (step time falls 20 %% over the first 200 steps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short untimed-region runs of the other configurations")
    ap.add_argument("--cpu-heads", type=int, default=0, help="heads the oracle is timed on (0 = auto)")
    ap.add_argument("--cold", action="store_true",
                    help="rotate over enough Q/K/V/O sets that every step reads from HBM (not the headline)")
    ap.add_argument("--dense-device-mask", action="store_true",
                    help="build the plan from a dense byte mask that lives in device memory (packed to bits by "
                         "the GPU) instead of from the pattern description; plan_ms then covers that path")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (outside the timed region) so that "
                         "rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE can be scaled against known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; every (batch, head) pair is independent, so a "
              "multi-GPU run would only split heads with no exchange. Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2506_06095_amd as smha
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    c = W.config(args.config)
    scattered = None
    if args.scattered > 0:
        c = W.scaled(W.config(3), name="scattered_2048_k%d" % args.scattered, seed=31, mask=None)
        scattered = W.scattered_spec(c.S, args.scattered, 3)     # dense [1][1][S][S]
    B, H, S, d = c.B, c.H, c.S, c.d
    Q, K, V = W.qkv_bits(B, H, S, d, c.dtype, c.std, c.seed)
    tdt = torch.float16 if c.dtype == "f16" else torch.bfloat16
    q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(tdt) for x in (Q, K, V))
    out = torch.empty_like(q)
    sets = [(q, k, v, out)]
    if args.cold:  # working set well beyond the 256 MB Infinity Cache + L2
        per_set = 4 * q.numel() * q.element_size()
        for _ in range(max(2, int(1.5e9 // per_set))):
            sets.append(tuple(t.clone() for t in (q, k, v, out)))

    force = {"auto": smha.SMHA_KERNEL_AUTO, "row": smha.SMHA_KERNEL_ROW, "block": smha.SMHA_KERNEL_BLOCK}[args.kernel]
    if scattered is not None:
        t0 = time.perf_counter()
        plan = smha.Plan.from_dense(scattered, block=c.block, head_dim=d, force=force, block_form=args.block_form)
        plan_ms = (time.perf_counter() - t0) * 1e3
    elif args.dense_device_mask:
        dense = W.dense_mask(c.mask, B, H, S)
        dev_mask = torch.from_numpy(dense).cuda()
        smha.Plan.from_dense(dev_mask, block=c.block, head_dim=d, force=force, block_form=args.block_form).close()   # warm-up (first launch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan = smha.Plan.from_dense(dev_mask, block=c.block, head_dim=d, force=force, block_form=args.block_form)
        plan_ms = (time.perf_counter() - t0) * 1e3
        del dev_mask, dense
    else:
        t0 = time.perf_counter()
        plan = smha.Plan.from_desc(c.mask, B, H, S, block=c.block, head_dim=d, force=force, block_form=args.block_form)
        plan_ms = (time.perf_counter() - t0) * 1e3
    info = plan.info()
    n_masks = info["Bm"] * info["Hm"]
    pairs_per_mask = B * H // n_masks
    nnz_flops = 4.0 * info["nnz"] * pairs_per_mask * d
    tile_flops = 4.0 * info["n_tiles64"] * 64 * 64 * pairs_per_mask * d
    if info["n_gathered"] > 0:
        # gathered tiles stand in for many sparse tiles: the kernel then executes at most two tiles' worth of
        # MFMA work per staged tile (one per 64-row half of a group), which is what the roofline may count
        tile_flops = min(tile_flops, 2.0 * 4.0 * info["n_union"] * 64 * 64 * pairs_per_mask * d)
    kernel = "row" if info["kernel"] == smha.SMHA_KERNEL_ROW else "block"

    stream = torch.cuda.current_stream()
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    def prewarm(fn, ms):
        # untimed: keep the GPU busy until its clocks have settled
        t_end = time.perf_counter() + ms * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()

    prewarm(lambda: plan.forward(q, k, v, out=out), args.prewarm_ms)
    for i in range(args.warmup):
        a = sets[i % len(sets)]
        plan.forward(a[0], a[1], a[2], out=a[3])
    torch.cuda.synchronize()
    # Timed region: exactly `steps` forwards between two events on the launch stream (an event
    # between every two steps would put a ~6 us bubble after each: the next kernel waits for the
    # event's own packet), bracketed by synchronisations; wall clock around the same region.
    ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_a.record(stream)
    for i in range(args.steps):
        a = sets[(args.warmup + i) % len(sets)]
        plan.forward(a[0], a[1], a[2], out=a[3])
    ev_b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    launch_ms = ev_a.elapsed_time(ev_b) / args.steps  # GPU time per step over the timed region
    # Spread of single launches, outside the timed region: one event pair per step.  Not the same
    # quantity as launch_ms: short workloads carry the event's own latency here, long ones run a
    # little faster than in the timed region (the bubbles are idle time, and the chip clocks higher).
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record(stream)
    for i in range(args.steps):
        a = sets[(args.warmup + i) % len(sets)]
        plan.forward(a[0], a[1], a[2], out=a[3])
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])  # ms per launch

    if kernel == "block":
        achieved = tile_flops / (launch_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[c.dtype], "unit": "TFLOP/s",
                "frac": achieved / PEAK_TFLOPS[c.dtype], "traffic": None,
                "kernel": smha.smha_kernel_name(plan.handle, d, 0 if c.dtype == "f16" else 1),
                "flops_per_launch": tile_flops, "launch_ms": launch_ms,
                "compulsory_hbm_bytes": 4.0 * B * H * S * d * 2}
    else:
        # Q + O once, every K/V row once, 4 bytes per unmasked entry of index, row pointers
        alg_bytes = 4.0 * B * H * S * d * 2 + 4.0 * info["nnz"] + 4.0 * (S + 1) * n_masks
        achieved = alg_bytes / (launch_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                "kernel": smha.smha_kernel_name(plan.handle, d, 0 if c.dtype == "f16" else 1),
                "bytes_per_launch": alg_bytes, "launch_ms": launch_ms}

    tr = MEASURED_TRAFFIC.get((c.name, roof["kernel"]))
    if tr is not None:
        roof["traffic"] = tr["read_bytes"] + tr["write_bytes"]
        roof["traffic_detail"] = dict(tr, unit="bytes per launch",
                                      source="constants in bench.py, copied from the rocprofv3 --pmc summaries under profiles/ "
                                             "(not measured by this run)")
    result = {
        "metric": "masked-MHA effective TFLOP/s over unmasked entries (latency in ms_per_step)",
        "value": nnz_flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "prewarm_ms": args.prewarm_ms, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": c.dtype,
        "data": "synthetic",
        "config": {"workload": c.name, "B": B, "H": H, "S": S, "d": d, "block": c.block,
                   "kernel": kernel, "nnz_per_step": info["nnz"] * pairs_per_mask,
                   "tiles64_per_step": info["n_tiles64"] * pairs_per_mask,
                   "kernel_steps_per_step": info["n_union"] * pairs_per_mask,
                   "gathered_tiles_per_step": info["n_gathered"] * pairs_per_mask,
                   "plan_from": "dense host mask" if scattered is not None else
                                "dense device mask" if args.dense_device_mask else "pattern description",
                   "cache": "cold (%d rotating sets)" % len(sets) if args.cold else "hot"},
        "latency_ms": {"timed_region_mean": launch_ms, "single_launch_mean": float(per.mean()),
                       "single_launch_median": float(np.median(per)), "single_launch_min": float(per.min())},
        "tile_tflops": tile_flops / (launch_ms * 1e-3) / 1e12,
        "plan_ms": plan_ms,
        "roofline": roof,
    }

    if not args.no_other_configs:
        # the other configurations, outside the timed region: latency of the selected kernel (mean of 30 launches)
        others = {}
        for idx in (1, 2, 3, 4, 5):
            if idx == args.config:
                continue
            oc = W.config(idx)
            odt = torch.float16 if oc.dtype == "f16" else torch.bfloat16
            g = torch.Generator(device="cuda").manual_seed(oc.seed)
            oq, ok_, ov = (torch.randn(oc.B, oc.H, oc.S, oc.d, device="cuda", generator=g).mul_(oc.std).to(odt) for _ in range(3))
            oo = torch.empty_like(oq)
            with smha.Plan.from_desc(oc.mask, oc.B, oc.H, oc.S, block=oc.block, head_dim=oc.d) as op:
                oi = op.info()
                prewarm(lambda: op.forward(oq, ok_, ov, out=oo), min(args.prewarm_ms, 40.0))
                for _ in range(5):
                    op.forward(oq, ok_, ov, out=oo)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(30):
                    op.forward(oq, ok_, ov, out=oo)
                e1.record(stream)
                torch.cuda.synchronize()
                oms = e0.elapsed_time(e1) / 30
            onnz = oi["nnz"] * (oc.B * oc.H // (oi["Bm"] * oi["Hm"]))
            others[oc.name] = {"ms": oms, "kernel": "row" if oi["kernel"] == smha.SMHA_KERNEL_ROW else "block",
                               "effective_tflops": 4.0 * onnz * oc.d / (oms * 1e-3) / 1e12}
            del oq, ok_, ov, oo
        result["other_configs"] = others

    if not args.no_cpu_baseline:
        import oracle
        masks = scattered if scattered is not None else W.dense_mask(c.mask, B, H, S)
        Bm, Hm = masks.shape[:2]
        flat = [(b, h) for b in range(B) for h in range(H)]
        n_heads = args.cpu_heads or max(1, min(len(flat), int(round(1.0e12 / (nnz_flops / len(flat))))))
        step = max(1, len(flat) // n_heads)
        sample = flat[::step][:n_heads]
        got = out.float().cpu().numpy()
        cpu_s, worst_abs, num, den = 0.0, 0.0, 0.0, 0.0
        flops = 0.0
        for (b, h) in sample:
            m1 = np.ascontiguousarray(masks[b if Bm > 1 else 0, h if Hm > 1 else 0][None, None])
            sl = [np.ascontiguousarray(x[b:b + 1, h:h + 1]) for x in (Q, K, V)]
            t1 = time.perf_counter()
            ref = oracle.masked_attention(*sl, c.dtype, m1)
            cpu_s += time.perf_counter() - t1
            flops += 4.0 * float(m1.sum()) * d
            diff = got[b, h].astype(np.float64) - ref[0, 0]
            worst_abs = max(worst_abs, float(np.abs(diff).max()))
            num += float((diff ** 2).sum())
            den += float((ref ** 2).sum())
        result["cpu_baseline"] = {"value": flops / cpu_s / 1e12, "unit": "TFLOP/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"{len(sample)} of {len(flat)} (batch, head) pairs of {c.name}, "
                                            f"full sequence, {cpu_s:.1f} s"}
        result["parity_on_sample"] = {"max_abs": worst_abs, "rel_fro": (num / max(den, 1e-300)) ** 0.5}
    plan.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
