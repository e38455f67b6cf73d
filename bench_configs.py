#!/usr/bin/env python3
"""Forward + backward time of every projection of the five benchmark configurations (the tiny fp32
case, Llama-2-7B q_proj, Llama-2-7B MLP, the Llama-2-13B layer, the Llama-2-70B MLP stage share),
through the same library calls as bench.py, inputs resident in HBM.

Prints one JSON line per (configuration, projection): HIP-event time of `--iters` forward +
backward pairs after `--warmup` pairs, useful TFLOP/s (4 T h d + 6 sum t_k r_k (h + d)), tokens/s
and the share of the 2.5 PFLOP/s dense bf16 MFMA peak.  With --md the same figures are printed as a
markdown table (the form kept under profiles/).  A side table: bench.py is the benchmark proper.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--md", action="store_true", help="print a markdown table instead of JSON lines")
    args = ap.parse_args()

    import torch
    from paper_2312_02515_amd import binding as mb
    from paper_2312_02515_amd import workloads as wl

    assert torch.cuda.is_available(), "bench_configs.py needs a GPU"
    dev = "cuda:0"
    rows = []
    for ci, name in enumerate(wl.WORKLOAD_ORDER):
        w = wl.WORKLOADS[name]
        for pi, p in enumerate(w.projections):
            inp = wl.make_workload_inputs(w, pi, device=dev, seed=args.seed)
            prob = mb.Problem(w.T, p.h, p.d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
            saved, ws = prob.alloc_saved(), prob.alloc_workspace()
            Y = torch.empty((w.T, p.d), dtype=inp.X.dtype, device=dev)
            dX = torch.empty((w.T, p.h), dtype=inp.X.dtype, device=dev)
            dA, dB = prob.alloc_grads()

            def pair():
                mb.mlora_lora_fwd(prob, inp.X, Y, saved, ws)
                mb.mlora_lora_bwd(prob, inp.X, inp.dY, saved, dX, dA, dB, False, ws)

            for _ in range(args.warmup):
                pair()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.iters):
                pair()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1) / args.iters
            tf = w.flops(p) / ms / 1e9
            rec = {"config": ci + 1, "workload": name, "projection": p.name, "h": p.h, "d": p.d, "T": w.T, "K": w.K,
                   "dtype": w.dtype, "kernel_path": prob.kernel_path(), "ms": ms, "tflops": tf,
                   "tokens_per_s": w.T / (ms * 1e-3), "pct_of_bf16_mfma_peak": 100.0 * tf / PEAK_BF16_TFLOPS}
            rows.append(rec)
            if not args.md:
                print(json.dumps(rec), flush=True)
            del inp, prob, saved, ws, Y, dX, dA, dB
            torch.cuda.empty_cache()
    if args.md:
        print("| Config | Workload | Projection (h -> d) | T | K | kernels | ms fwd+bwd | useful TFLOP/s | tokens/s | % of 2.5 PFLOP/s |")
        print("|---|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            kern = "MFMA" if r["kernel_path"] == 0 else "generic (fp32 mode)"
            pct = f'{r["pct_of_bf16_mfma_peak"]:.1f}' if r["dtype"] == "bf16" else "-"
            print(f'| {r["config"]} | {r["workload"]} | {r["projection"]} ({r["h"]} -> {r["d"]}) | {r["T"]} | {r["K"]} | {kern} '
                  f'| {r["ms"]:.3f} | {r["tflops"]:.1f} | {r["tokens_per_s"]:.3e} | {pct} |')


if __name__ == "__main__":
    main()
