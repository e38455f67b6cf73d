#!/usr/bin/env python3
"""Projections that share their input (q, k, v of an attention block; gate, up of an MLP):
the group entry points against one call per projection, on the Llama-2-13B layer shapes of
bench.py's workload (T = 32768, 16 adapters of ranks {8,16,32,64}).

  group     mlora_lora_group_fwd + mlora_lora_group_bwd: X is streamed once for all Z_p and once
            for all dA_p; one kernel accumulates dX = sum_p (dY_p W_p^T + ...) in fp32
  separate  mlora_lora_fwd + mlora_lora_bwd per projection, each writing its own dX_p, then
            dX = sum_p dX_p with elementwise adds (what an autograd engine does with the
            single-projection operator)

Prints one JSON line per group with the median time of each mode.  A side experiment:
bench.py is the benchmark proper.
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
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()

    import torch
    from paper_2312_02515_amd import binding as mb
    from paper_2312_02515_amd import workloads as wl

    assert torch.cuda.is_available(), "bench_groups.py needs a GPU"
    dev = "cuda:0"
    w = wl.WORKLOADS["llama2_13b_layer"]
    for name, members in (("qkv", [0, 1, 2]), ("gate_up", [4, 5])):
        ins = [wl.make_workload_inputs(w, pi, device=dev, seed=args.seed) for pi in members]
        X = ins[0].X
        T, h = X.shape
        probs = [mb.Problem(T, h, i.W.shape[1], i.W, i.seg_offsets, i.ranks, i.scalings, i.A, i.B) for i in ins]
        group = mb.Group(probs)
        saved = [p.alloc_saved() for p in probs]
        gws = group.alloc_workspace()
        wss = [p.alloc_workspace() for p in probs]
        Y = [torch.empty((T, i.W.shape[1]), dtype=X.dtype, device=dev) for i in ins]
        dX = torch.empty((T, h), dtype=X.dtype, device=dev)
        dXp = [torch.empty((T, h), dtype=X.dtype, device=dev) for _ in ins]
        grads = [p.alloc_grads() for p in probs]
        dA, dB = [g[0] for g in grads], [g[1] for g in grads]
        dYs = [i.dY for i in ins]

        def grouped():
            mb.mlora_lora_group_fwd(group, X, Y, saved, gws)
            mb.mlora_lora_group_bwd(group, X, dYs, saved, dX, dA, dB, False, gws)

        def separate():
            for p, pr in enumerate(probs):
                mb.mlora_lora_fwd(pr, X, Y[p], saved[p], wss[p])
            for p, pr in enumerate(probs):
                mb.mlora_lora_bwd(pr, X, dYs[p], saved[p], dXp[p], dA[p], dB[p], False, wss[p])
            torch.add(dXp[0], dXp[1], out=dX)
            for t in dXp[2:]:
                dX.add_(t)

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

        tg, ts = timed(grouped), timed(separate)
        flops = sum(w.flops(w.projections[pi]) for pi in members)
        print(json.dumps({"group": name, "projections": [w.projections[pi].name for pi in members], "T": T,
                          "group_ms": tg, "separate_ms": ts, "separate_over_group": ts / tg,
                          "group_tflops": flops / tg / 1e9, "separate_tflops": flops / ts / 1e9}), flush=True)
        del ins, probs, group, saved, gws, wss, Y, dX, dXp, grads, dA, dB, dYs


if __name__ == "__main__":
    main()
