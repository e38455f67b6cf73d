"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI,
run the CPU oracle on the same bit patterns, compare by relative Frobenius error.

What is compared (tolerance 2e-2 in bf16 mode, 1e-5 in fp32 mode, never loosened):
  * Y and dX as whole tensors,
  * Y and dX per row block: each task's rows on their own, and the rows before the first
    and after the last task (base term only) on their own -- one norm over the whole tensor
    would let a single task's LoRA term (a few per cent of the tensor) vanish unnoticed,
  * every dA_k and dB_k on its own.
With W = 0 the row blocks of Y and dX *are* the LoRA terms of Eq. "forward" and
Eq. "grad_output", so the same tolerance then applies to those terms directly
(`zero_base_weight`).  The checkers take device or host tensors, so the CPU-only tests
can feed them deliberately wrong "outputs" built from the oracle and see them fail.
"""
import numpy as np
import torch

from oracle import batchlora_oracle as orc

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-5}

# Shapes the MFMA kernels take (h, d multiples of 64, ranks multiples of 8), ragged in every
# other way: T, h, d, tokens, ranks, lead.  Shared by the GPU tests and by the CPU test that
# checks the checker's sensitivity on the same inputs.
MFMA_SMALL_CASES = [
    (1000, 192, 320, [100, 0, 333, 500], [8, 24, 128, 64], 7),        # rank 128, empty segment, tails
    (900, 128, 64, [130, 700], [16, 8], 3),                           # narrow output, small ranks
    (1537, 448, 576, [1, 255, 257, 1024], [64, 32, 8, 16], 0),        # one-token task, tile-straddling tasks
]
# Cases run with W = 0 (the outputs are the LoRA terms alone)
LORA_TERM_CASES = MFMA_SMALL_CASES + [
    (1300, 256, 384, [1, 300, 211, 512, 40], [8, 128, 8, 64, 16], 100),  # rank 8 beside rank 128, lead and tail rows
    (2048, 128, 256, [250, 12, 500, 6, 1000], [16, 8, 32, 8, 24], 130),  # tasks inside and across 256-row tiles
    (700, 320, 192, [31, 33, 95, 97, 160, 161], [8, 16, 8, 16, 8, 16], 17),  # boundaries inside 32-row fragments
]


def np64(t) -> np.ndarray:
    if isinstance(t, np.ndarray):
        return t.astype(np.float64, copy=False)
    return t.detach().to("cpu").to(torch.float64).numpy()


def relerr(got: np.ndarray, ref: np.ndarray, zero_scale: float = 1.0) -> float:
    n = float(np.linalg.norm(ref))
    e = float(np.linalg.norm(got - ref))
    return e / n if n > 0 else e / zero_scale


def row_blocks(seg_offsets, T):
    """Named row ranges that partition [0, T): 'lead', 'task0', ..., 'tail' (empty ones left out)."""
    off = [int(o) for o in seg_offsets] if len(seg_offsets) else [0]
    blocks = []
    if off[0] > 0:
        blocks.append(("lead", 0, off[0]))
    for k in range(len(off) - 1):
        if off[k + 1] > off[k]:
            blocks.append((f"task{k}", off[k], off[k + 1]))
    if off[-1] < T:
        blocks.append(("tail", off[-1], T))
    return blocks


def zero_base_weight(inp):
    """The same problem with W = 0: Y and dX are then the LoRA terms alone."""
    inp.W.zero_()
    return inp


def run_hip(inp, accumulate=False, want_dx=True, preset_grads=None, poison=True, recompute=False):
    """Forward + backward through the binding (the activation-recompute pair of entry points if
    `recompute`).  Returns dict of device tensors."""
    from paper_2312_02515_amd import binding as mb
    dev = inp.X.device
    T, h = inp.X.shape
    d = inp.W.shape[1]
    prob = mb.Problem(T, h, d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
    saved = prob.alloc_saved()
    ws = prob.alloc_recompute_workspace() if recompute else prob.alloc_workspace()
    Y = torch.empty((T, d), dtype=inp.X.dtype, device=dev)
    dX = torch.empty((T, h), dtype=inp.X.dtype, device=dev) if want_dx else None
    dA, dB = prob.alloc_grads()
    if poison:
        # unwritten outputs show up as NaN
        Y.fill_(float("nan"))
        if dX is not None:
            dX.fill_(float("nan"))
        saved.fill_(0xFF)
        ws.fill_(0xFF)
        for t in dA + dB:
            t.fill_(float("nan"))
    if preset_grads is not None:
        for t, v in zip(dA, preset_grads[0]):
            t.copy_(v)
        for t, v in zip(dB, preset_grads[1]):
            t.copy_(v)
    if recompute:
        mb.mlora_lora_fwd_nosave(prob, inp.X, Y, ws)
    else:
        mb.mlora_lora_fwd(prob, inp.X, Y, saved, ws)
    if poison:
        ws.fill_(0xFF)  # the workspace carries nothing between the two calls
    if recompute:
        mb.mlora_lora_bwd_recompute(prob, inp.X, inp.dY, dX, dA, dB, accumulate, ws)
    else:
        mb.mlora_lora_bwd(prob, inp.X, inp.dY, saved, dX, dA, dB, accumulate, ws)
    torch.cuda.synchronize()
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB}


def oracle_full(inp):
    X, W, dY = np64(inp.X), np64(inp.W), np64(inp.dY)
    A = [np64(a) for a in inp.A]
    B = [np64(b) for b in inp.B]
    H, _ = orc.forward(X, W, inp.seg_offsets, A, B, inp.scalings)
    dX, dA, dB = orc.backward(X, W, dY, inp.seg_offsets, A, B, inp.scalings)
    return {"Y": H, "dX": dX, "dA": dA, "dB": dB}


def block_errors(name, got, ref, seg_offsets):
    """Relative error of the whole tensor and of every row block of it."""
    errs = {name: relerr(got, ref)}
    for bname, lo, hi in row_blocks(seg_offsets, ref.shape[0]):
        # an all-zero reference block (e.g. uncovered rows when W = 0) must come out as zeros
        errs[f"{name}[{bname}]"] = relerr(got[lo:hi], ref[lo:hi])
    return errs


def check_full(inp, out, tol, want_dx=True, label="", ref=None):
    ref = oracle_full(inp) if ref is None else ref
    errs = block_errors("Y", np64(out["Y"]), ref["Y"], inp.seg_offsets)
    if want_dx:
        errs.update(block_errors("dX", np64(out["dX"]), ref["dX"], inp.seg_offsets))
    for k in range(len(inp.ranks)):
        errs[f"dA{k}"] = relerr(np64(out["dA"][k]), ref["dA"][k])
        errs[f"dB{k}"] = relerr(np64(out["dB"][k]), ref["dB"][k])
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"{label}: relative Frobenius error above {tol}: {bad}"
    return errs


def row_errors(name, got, ref, rows):
    """Relative error of every sampled row on its own (rows of Y and dX are independent results)."""
    num = np.linalg.norm(got - ref, axis=1)
    den = np.linalg.norm(ref, axis=1)
    e = np.where(den > 0, num / np.where(den > 0, den, 1.0), num)
    worst = int(np.argmax(e)) if e.size else 0
    return {name: relerr(got, ref), f"{name}[worst row {int(rows[worst]) if e.size else -1}]": float(e.max()) if e.size else 0.0}


def check_sampled(inp, out, tol, rows, grad_adapters=None, label=""):
    """Complete rows of Y and dX for the sampled `rows`, each row held to the tolerance on its
    own; whole dA_k, dB_k for the adapters in `grad_adapters` (default: all)."""
    T = inp.X.shape[0]
    W = np64(inp.W)
    A = [np64(a) for a in inp.A]
    B = [np64(b) for b in inp.B]
    rs, off2 = orc.gather_rows_problem(rows, inp.seg_offsets, T)
    idx = torch.as_tensor(rs, device=inp.X.device)
    Xs, dYs = np64(inp.X[idx]), np64(inp.dY[idx])
    H, _ = orc.forward(Xs, W, off2, A, B, inp.scalings)
    dXr, _, _ = orc.backward(Xs, W, dYs, off2, A, B, inp.scalings)
    errs = row_errors("Y", np64(out["Y"][idx]), H, rs)
    errs.update(row_errors("dX", np64(out["dX"][idx]), dXr, rs))
    del W
    ks = range(len(inp.ranks)) if grad_adapters is None else grad_adapters
    for k in ks:
        lo, hi = inp.seg_offsets[k], inp.seg_offsets[k + 1]
        ga, gb = orc.adapter_gradients(np64(inp.X[lo:hi]), np64(inp.dY[lo:hi]), A[k], B[k], inp.scalings[k])
        errs[f"dA{k}"] = relerr(np64(out["dA"][k]), ga)
        errs[f"dB{k}"] = relerr(np64(out["dB"][k]), gb)
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"{label}: relative Frobenius error above {tol}: {bad}"
    return errs
