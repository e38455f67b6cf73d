#!/usr/bin/env python3
"""Benchmark of the BatchLoRA multi-adapter LoRA linear operator on one MI355X.

One "step" = forward of all seven LoRA-wrapped projections of a Llama-2-13B decoder
layer (q, k, v, o, gate, up, down; K = 16 adapters of ranks {8,16,32,64}, 2048 tokens
each, 32768 tokens in all), then the seven backward passes in reverse order, each
projection with its own seeded synthetic X and dY, all on one stream.  Inputs are
resident in HBM before the timed region starts.

Prints ONE JSON line:
  metric/value   useful TFLOP/s of the whole step (4 T h d + 6 sum t_k r_k (h+d) per projection)
  roofline       the MFMA base-product kernel against the dense bf16 MFMA peak, from HIP events the
                 library records on the launch stream around each of its launches, in a pass of
                 its own after the timed region (the timed steps run without those events)
  roofline_lowrank  the same for the four HBM-bound low-rank kernels against the HBM peak
  cpu_baseline   the CPU fp64 oracle timed on this machine's host cores on a bounded token sample
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
WORKLOAD = "llama2_13b_layer"


def _traffic_bytes_per_launch():
    """Bytes per launch that the dominant kernel's L2 misses request from the memory side
    (FETCH_SIZE + WRITE_SIZE), from the committed rocprofv3 counter runs of this same command
    (profiles/gemm_traffic.json); (None, None) if that summary is absent.  Counters cannot be read
    inside this process, so the figure belongs to the kernel build the summary names."""
    p = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    try:
        with open(p) as f:
            d = json.load(f)
            return d.get("hbm_bytes_per_launch_avg"), d.get("source")
    except (OSError, ValueError):
        return None, None


def sample_power(run_steps, seconds=2.0):
    """Socket power and shader clock while the hot path runs (outside the timed region): keeps
    launching steps for `seconds` while a thread polls `amd-smi metric -p -c`.  Returns None if
    amd-smi is not available.  Context for the roofline: at the board's power cap the matrix
    cores run below the 2.4 GHz the published peak assumes."""
    import re
    import shutil
    import subprocess
    import threading
    import torch
    if shutil.which("amd-smi") is None:
        return None
    samples, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            try:
                out = subprocess.run(["amd-smi", "metric", "-p", "-c"], capture_output=True, text=True, timeout=10).stdout
            except Exception:
                return
            pw = re.search(r"SOCKET_POWER:\s*([0-9.]+)\s*W", out)
            gfx = out.split("GFX_0:")[1] if "GFX_0:" in out else ""
            clks = [float(x) for x in re.findall(r"\n\s+CLK:\s*([0-9.]+)\s*MHz", gfx)[:8]]
            if pw and clks:
                samples.append((float(pw.group(1)), sum(clks) / len(clks)))

    th = threading.Thread(target=poll, daemon=True)
    th.start()
    t_end = time.perf_counter() + seconds
    while time.perf_counter() < t_end:
        run_steps()
        torch.cuda.synchronize()
    stop.set()
    th.join(timeout=15)
    samples = samples[1:] if len(samples) > 1 else samples  # the first poll may predate the load
    if not samples:
        return None
    return {"socket_power_w": sum(p for p, _ in samples) / len(samples),
            "gfx_clock_mhz": sum(c for _, c in samples) / len(samples), "samples": len(samples),
            "source": "amd-smi metric -p -c, polled while the step loop runs after the timed region"}


def cpu_baseline(wl_mod, w, tokens_per_adapter, seed):
    """Time the oracle (as it stands) on the first `tokens_per_adapter` tokens of every adapter,
    all seven projections, forward + backward."""
    import numpy as np
    import torch
    from oracle import batchlora_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    K = w.K
    off = [i * tokens_per_adapter for i in range(K + 1)]
    Ts = off[-1]
    total_flops, total_s = 0.0, 0.0
    for pi, p in enumerate(w.projections):
        inp = wl_mod.make_inputs(Ts, p.h, p.d, off, w.ranks, w.scalings, w.torch_dtype(), device="cpu",
                                 seed=seed, sigma_w=w.sigma_w, proj_id=pi)
        X, W, dY = (t.to(torch.float64).numpy() for t in (inp.X, inp.W, inp.dY))
        A = [a.to(torch.float64).numpy() for a in inp.A]
        B = [b.to(torch.float64).numpy() for b in inp.B]
        t0 = time.perf_counter()
        orc.forward(X, W, off, A, B, inp.scalings)
        orc.backward(X, W, dY, off, A, B, inp.scalings)
        total_s += time.perf_counter() - t0
        total_flops += orc.flops(Ts, p.h, p.d, off, w.ranks)
    return {"value": total_flops / total_s / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "implementation": "numpy float64; every product of the equations is one multithreaded BLAS dgemm",
            "tokens_per_s": Ts / total_s, "seconds": total_s,
            "sample": f"first {tokens_per_adapter} tokens of each of the {K} adapters ({Ts} of {w.T} tokens), "
                      f"all 7 projections, fp64 forward+backward"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-tokens", type=int, default=512, help="tokens per adapter in the CPU oracle sample (0 = skip)")
    ap.add_argument("--no-power", action="store_true", help="skip the amd-smi power/clock sample after the timed region")
    ap.add_argument("--recompute", action="store_true",
                    help="time the activation-recompute pair of entry points (nothing saved between forward and "
                         "backward; the backward recomputes s x A) instead of the default pair")
    ap.add_argument("--w8", action="store_true",
                    help="time the 8-bit-weight pair of entry points (the frozen weight is handed over as int8 "
                         "codes + per-column scales and decoded inside every call) instead of the default pair")
    ap.add_argument("--kernel-path", type=int, default=0,
                    help="test switch of include/mlora_testing.h (bit mask; 0 = the fastest kernels)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="before the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "traffic that calibrates the FETCH_SIZE / WRITE_SIZE counters in rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build is single-GPU by design (no collectives, no sharding); "
                         "run it with --gpus 1.\n")
        sys.exit(2)

    import torch
    from paper_2312_02515_amd import binding as mb
    from paper_2312_02515_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[WORKLOAD]
    stream = torch.cuda.current_stream()
    if args.kernel_path:
        mb.set_kernel_path(args.kernel_path)

    projs = []
    for pi, p in enumerate(w.projections):
        inp = wl.make_workload_inputs(w, pi, device=dev, seed=args.seed)
        prob = mb.Problem(w.T, p.h, p.d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
        dA, dB = prob.alloc_grads()
        if args.w8:
            Wq, c = mb.mlora_w8_quantize(inp.W)
            torch.cuda.synchronize()
            inp.W = None                   # the bf16 weight is gone: only its code stays resident
            prob = mb.Problem(w.T, p.h, p.d, None, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B,
                              dtype=inp.X.dtype, device=dev)
        projs.append(dict(p=p, inp=inp, prob=prob, saved=prob.alloc_saved(), Wq=Wq if args.w8 else None,
                          c=c if args.w8 else None,
                          ws=prob.alloc_w8_workspace() if args.w8 else
                          prob.alloc_recompute_workspace() if args.recompute else prob.alloc_workspace(),
                          Y=torch.empty((w.T, p.d), dtype=inp.X.dtype, device=dev),
                          dX=torch.empty((w.T, p.h), dtype=inp.X.dtype, device=dev), dA=dA, dB=dB))
    flops_step = sum(w.flops(p) for p in w.projections)

    def step():
        if args.recompute:
            for q in projs:
                mb.mlora_lora_fwd_nosave(q["prob"], q["inp"].X, q["Y"], q["ws"], stream)
            for q in reversed(projs):
                mb.mlora_lora_bwd_recompute(q["prob"], q["inp"].X, q["inp"].dY, q["dX"], q["dA"], q["dB"], False,
                                            q["ws"], stream)
            return
        if args.w8:
            for q in projs:
                mb.mlora_lora_fwd_w8(q["prob"], q["Wq"], q["c"], q["inp"].X, q["Y"], q["saved"], q["ws"], stream)
            for q in reversed(projs):
                mb.mlora_lora_bwd_w8(q["prob"], q["Wq"], q["c"], q["inp"].X, q["inp"].dY, q["saved"], q["dX"],
                                     q["dA"], q["dB"], False, q["ws"], stream)
            return
        for q in projs:
            mb.mlora_lora_fwd(q["prob"], q["inp"].X, q["Y"], q["saved"], q["ws"], stream)
        for q in reversed(projs):
            mb.mlora_lora_bwd(q["prob"], q["inp"].X, q["inp"].dY, q["saved"], q["dX"], q["dA"], q["dB"], False,
                              q["ws"], stream)

    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # per-kernel durations: the same steps once more, each launch bracketed by HIP events
    prof_steps = min(args.steps, 5)
    mb.profile_kernels(True)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    mb.profile_kernels(False)
    prof = mb.profile_kernels_read()
    gemm_ms, gemm_flops, gemm_launches = prof["gemm"]

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    traffic, traffic_src = _traffic_bytes_per_launch()
    out = {
        "metric": "multi-adapter LoRA linear fwd+bwd TFLOP/s",
        "value": tflops, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD, "tokens": w.T, "adapters": w.K, "ranks": list(w.ranks),
                   "projections": [f"{p.name}:{p.h}x{p.d}" for p in w.projections], "seed": args.seed,
                   "variant": "w8" if args.w8 else "recompute" if args.recompute else "saved"},
        "tokens_per_s": w.T / (ms_per_step * 1e-3),
        "pct_of_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "k_gemm_mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "launches": gemm_launches, "avg_launch_ms": gemm_ms / max(gemm_launches, 1),
                     "share_of_step_time": gemm_ms / prof_steps / ms_per_step,
                     "traffic": traffic, "traffic_source": traffic_src},
    }
    # the HBM-bound kernels (s x A and s dy B^T: "rows"; dA_k and dB_k: "grad"): algorithmic bytes per
    # launch (activations read once, results written once) over the HIP-event duration
    out["roofline_lowrank"] = {
        kind: {"bound": "hbm", "kernel": kname, "achieved": (by / (ms * 1e-3) / 1e9 if ms > 0 else 0.0),
               "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": (by / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS if ms > 0 else 0.0),
               "launches": n, "avg_launch_ms": ms / max(n, 1), "share_of_step_time": ms / prof_steps / ms_per_step}
        for kind, kname, (ms, by, n) in (("rows", "k_lowrank_mfma", prof["rows"]), ("grad", "k_grad_mfma", prof["grad"]))}
    if not args.no_power:
        out["power"] = sample_power(step)
    if args.cpu_tokens > 0:
        out["cpu_baseline"] = cpu_baseline(wl, w, args.cpu_tokens, args.seed)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
