"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI,
run the CPU oracle on the same bit patterns, compare by relative Frobenius error."""
import numpy as np
import torch

from oracle import batchlora_oracle as orc

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-5}


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def relerr(got: np.ndarray, ref: np.ndarray, zero_scale: float = 1.0) -> float:
    n = float(np.linalg.norm(ref))
    e = float(np.linalg.norm(got - ref))
    return e / n if n > 0 else e / zero_scale


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


def check_full(inp, out, tol, want_dx=True, label=""):
    ref = oracle_full(inp)
    errs = {"Y": relerr(np64(out["Y"]), ref["Y"])}
    if want_dx:
        errs["dX"] = relerr(np64(out["dX"]), ref["dX"])
    for k in range(len(inp.ranks)):
        errs[f"dA{k}"] = relerr(np64(out["dA"][k]), ref["dA"][k])
        errs[f"dB{k}"] = relerr(np64(out["dB"][k]), ref["dB"][k])
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"{label}: relative Frobenius error above {tol}: {bad}"
    return errs


def check_sampled(inp, out, tol, rows, grad_adapters=None, label=""):
    """Full rows of Y and dX for the sampled `rows`; whole dA_k, dB_k for the
    adapters in `grad_adapters` (default: all)."""
    T = inp.X.shape[0]
    W = np64(inp.W)
    A = [np64(a) for a in inp.A]
    B = [np64(b) for b in inp.B]
    rs, off2 = orc.gather_rows_problem(rows, inp.seg_offsets, T)
    idx = torch.as_tensor(rs, device=inp.X.device)
    Xs, dYs = np64(inp.X[idx]), np64(inp.dY[idx])
    H, _ = orc.forward(Xs, W, off2, A, B, inp.scalings)
    dXr, _, _ = orc.backward(Xs, W, dYs, off2, A, B, inp.scalings)
    errs = {"Y": relerr(np64(out["Y"][idx]), H), "dX": relerr(np64(out["dX"][idx]), dXr)}
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
