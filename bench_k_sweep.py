#!/usr/bin/env python3
"""Launch-count experiment of the BatchLoRA operator (section 3.3.2 and the BatchLoRA ablation of
section 4.4): fixed total tokens T, K = 1 ... 64 adapters of equal share, rank 16.

  batched   one forward + one backward call of the library for all K tasks
            (the shared base product is launched once over all tokens)
  separate  K forward + K backward calls, each on one task's rows with its own adapter
            (the unbatched workflow: every task launches its own base product)

Both run through the same kernels of this library on one stream, inputs resident in HBM.
Prints one JSON line per (T, K) with the median time of each mode over `--iters` repetitions
and their ratio.  A side experiment: bench.py is the benchmark proper.
"""
import argparse
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, nargs="+", default=[8192, 32768])
    ap.add_argument("--features", type=int, default=4096, help="h = d (Llama-2-7B q_proj)")
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--adapters", type=int, nargs="+", default=[1, 2, 4, 8, 16, 32, 64])
    ap.add_argument("--iters", type=int, default=15)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--md", action="store_true", help="print a markdown table instead of JSON lines")
    args = ap.parse_args()
    rows = []

    import torch
    from paper_2312_02515_amd import binding as mb
    from paper_2312_02515_amd import workloads as wl

    assert torch.cuda.is_available(), "bench_k_sweep.py needs a GPU"
    dev = "cuda:0"
    h = d = args.features
    for T in args.tokens:
        for K in args.adapters:
            if T % K:
                continue
            t = T // K
            off = [k * t for k in range(K + 1)]
            ranks, scal = [args.rank] * K, [2.0] * K
            inp = wl.make_inputs(T, h, d, off, ranks, scal, torch.bfloat16, device=dev, seed=args.seed, sigma_w=0.02)
            Y = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
            dX = torch.empty((T, h), dtype=torch.bfloat16, device=dev)
            whole = mb.Problem(T, h, d, inp.W, off, ranks, scal, inp.A, inp.B)
            saved, ws = whole.alloc_saved(), whole.alloc_workspace()
            dA, dB = whole.alloc_grads()
            parts = []
            for k in range(K):
                p = mb.Problem(t, h, d, inp.W, [0, t], [args.rank], [2.0], [inp.A[k]], [inp.B[k]])
                parts.append((p, p.alloc_saved(), p.alloc_workspace(), slice(off[k], off[k + 1])))

            def batched():
                mb.mlora_lora_fwd(whole, inp.X, Y, saved, ws)
                mb.mlora_lora_bwd(whole, inp.X, inp.dY, saved, dX, dA, dB, False, ws)

            def separate():
                for k, (p, sv, w_, rows) in enumerate(parts):
                    mb.mlora_lora_fwd(p, inp.X[rows], Y[rows], sv, w_)
                for k, (p, sv, w_, rows) in enumerate(parts):
                    mb.mlora_lora_bwd(p, inp.X[rows], inp.dY[rows], sv, dX[rows], [dA[k]], [dB[k]], False, w_)

            def timed(fn):
                for _ in range(args.warmup):
                    fn()
                torch.cuda.synchronize()
                ms = []
                for _ in range(args.iters):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    fn()
                    e1.record()
                    e1.synchronize()
                    ms.append(e0.elapsed_time(e1))
                return statistics.median(ms)

            tb, ts = timed(batched), timed(separate)
            flops = 4.0 * T * h * d + 6.0 * T * args.rank * (h + d)
            rec = {"T": T, "K": K, "tokens_per_task": t, "h": h, "d": d, "rank": args.rank,
                   "batched_ms": tb, "separate_ms": ts, "separate_over_batched": ts / tb,
                   "batched_tflops": flops / tb / 1e9, "separate_tflops": flops / ts / 1e9}
            rows.append(rec)
            if not args.md:
                print(json.dumps(rec), flush=True)
            del inp, Y, dX, whole, saved, ws, dA, dB, parts
    if args.md:
        print("| T | K | tokens per task | batched ms | separate ms | separate / batched | batched TFLOP/s |")
        print("|---|---|---|---|---|---|---|")
        for r in rows:
            print(f'| {r["T"]} | {r["K"]} | {r["tokens_per_task"]} | {r["batched_ms"]:.3f} | {r["separate_ms"]:.3f} '
                  f'| {r["separate_over_batched"]:.2f} | {r["batched_tflops"]:.0f} |')


if __name__ == "__main__":
    main()
