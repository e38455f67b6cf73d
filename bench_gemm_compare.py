#!/usr/bin/env python3
"""The base product of the operator (K = 0: no adapters, so one call is one k_gemm_mfma launch)
beside the vendor's GEMM (torch.matmul, i.e. hipBLASLt) on the same box, shapes and data:

  * forward layout  Y  = X W     (W [h, d] row-major: "NN")
  * backward layout dX = dY W^T  (W [h, d] row-major: "NT")

on operands drawn like the benchmark's (X, dY ~ N(0,1), W ~ N(0, 0.02^2)), where the board runs at
its power cap, and on all-zero operands, where it does not; at the benchmark's size (T = 32768:
X is 320 MB, more than the 256 MB Infinity Cache) and at half of it (T = 16384: X, W and the
output of repeated launches stay cache-resident).  HIP-event time over `--iters` back-to-back
launches after `--warmup`.  Prints JSON lines, or a markdown table with --md.  A side
measurement: bench.py is the benchmark proper.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--md", action="store_true")
    args = ap.parse_args()

    import torch
    from paper_2312_02515_amd import binding as mb

    assert torch.cuda.is_available(), "bench_gemm_compare.py needs a GPU"
    dev = "cuda:0"

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.iters):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / args.iters

    rows = []
    for (T, h, d) in [(32768, 5120, 5120), (32768, 5120, 13824), (16384, 5120, 5120)]:
        for kind in ("random", "zeros"):
            g = torch.Generator(device=dev)
            g.manual_seed(T + h + d)

            def mk(shape, std):
                if kind == "zeros":
                    return torch.zeros(shape, device=dev, dtype=torch.bfloat16)
                return (torch.randn(shape, device=dev, dtype=torch.float32, generator=g) * std).to(torch.bfloat16)

            X, dY, W = mk((T, h), 1.0), mk((T, d), 1.0), mk((h, d), 0.02)
            Y = torch.empty((T, d), device=dev, dtype=torch.bfloat16)
            dX = torch.empty((T, h), device=dev, dtype=torch.bfloat16)
            flops = 2.0 * T * h * d
            prob = mb.Problem(T, h, d, W, [0], [], [], [], [])
            assert prob.kernel_path() == 0
            saved, ws = prob.alloc_saved(), prob.alloc_workspace()
            t = {
                "vendor_nn": timed(lambda: torch.matmul(X, W, out=Y)),
                "vendor_nt": timed(lambda: torch.matmul(dY, W.t(), out=dX)),
                "ours_nn": timed(lambda: mb.mlora_lora_fwd(prob, X, Y, saved, ws)),
                "ours_nt": timed(lambda: mb.mlora_lora_bwd(prob, X, dY, saved, dX, [], [], False, ws)),
            }
            rec = {"T": T, "h": h, "d": d, "operands": kind, "x_mb": T * h * 2 >> 20}
            rec.update({k + "_tflops": flops / v / 1e9 for k, v in t.items()})
            rows.append(rec)
            if not args.md:
                print(json.dumps(rec), flush=True)
            del X, dY, W, Y, dX, prob, saved, ws
            torch.cuda.empty_cache()
    if args.md:
        print("| T | h -> d | operands | X MB | vendor NN | this library NN | vendor NT | this library NT |")
        print("|---|---|---|---|---|---|---|---|")
        for r in rows:
            print(f'| {r["T"]} | {r["h"]} -> {r["d"]} | {r["operands"]} | {r["x_mb"]} | {r["vendor_nn_tflops"]:.0f} '
                  f'| {r["ours_nn_tflops"]:.0f} | {r["vendor_nt_tflops"]:.0f} | {r["ours_nt_tflops"]:.0f} |')


if __name__ == "__main__":
    main()
