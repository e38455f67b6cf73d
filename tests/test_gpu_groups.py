"""GPU parity of the projection-group entry points (several LoRA-wrapped projections fed by the
same X: q, k, v of an attention block; gate, up of an MLP) against the CPU fp64 oracle.
Tolerance as for the single calls: relative Frobenius error per output tensor <= 2e-2 (bf16),
<= 1e-5 (fp32)."""
import numpy as np
import pytest
import torch

from oracle import batchlora_oracle as orc
from paper_2312_02515_amd import workloads as wl
from tests.parity_util import TOL, block_errors, np64, relerr, row_errors

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _group_inputs(T, h, ds, tokens, ranks_per_p, dtype, lead=0, seed=0, sigma_w=None):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    assert off[-1] <= T
    sw = sigma_w if sigma_w is not None else 1.0 / np.sqrt(h)
    ins = []
    for p, (d, ranks) in enumerate(zip(ds, ranks_per_p)):
        scal = [0.75 + 0.5 * ((p + k) % 3) for k in range(len(ranks))]
        ins.append(wl.make_inputs(T, h, d, off, ranks, scal, dtype, device=DEV, seed=seed, sigma_w=sw, proj_id=p))
    for i in ins[1:]:
        i.X = ins[0].X  # the shared input
    return ins


def run_group(ins, accumulate=False, want_dx=True, preset=None, poison=True):
    from paper_2312_02515_amd import binding as mb
    X = ins[0].X
    T, h = X.shape
    probs = [mb.Problem(T, h, i.W.shape[1], i.W, i.seg_offsets, i.ranks, i.scalings, i.A, i.B) for i in ins]
    g = mb.Group(probs)
    saved = [p.alloc_saved() for p in probs]
    ws = g.alloc_workspace()
    Y = [torch.empty((T, i.W.shape[1]), dtype=X.dtype, device=DEV) for i in ins]
    dX = torch.empty((T, h), dtype=X.dtype, device=DEV) if want_dx else None
    grads = [p.alloc_grads() for p in probs]
    dA, dB = [g_[0] for g_ in grads], [g_[1] for g_ in grads]
    if poison:
        for t in Y + ([dX] if want_dx else []) + [t for l in dA + dB for t in l]:
            t.fill_(float("nan"))
        for t in saved + [ws]:
            t.fill_(0xFF)
    if preset is not None:
        for l in dA:
            for t in l:
                t.fill_(preset[0])
        for l in dB:
            for t in l:
                t.fill_(preset[1])
    mb.mlora_lora_group_fwd(g, X, Y, saved, ws)
    if poison:
        ws.fill_(0xFF)
    mb.mlora_lora_group_bwd(g, X, [i.dY for i in ins], saved, dX, dA, dB, accumulate, ws)
    torch.cuda.synchronize()
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB}


def check_group(ins, out, tol, label=""):
    X = np64(ins[0].X)
    Ws = [np64(i.W) for i in ins]
    dHs = [np64(i.dY) for i in ins]
    As = [[np64(a) for a in i.A] for i in ins]
    Bs = [[np64(b) for b in i.B] for i in ins]
    ss = [i.scalings for i in ins]
    off = ins[0].seg_offsets
    fw = orc.group_forward(X, Ws, off, As, Bs, ss)
    dX, dA, dB = orc.group_backward(X, Ws, dHs, off, As, Bs, ss)
    # whole tensors and every task's row block on its own (see tests/parity_util.py)
    errs = block_errors("dX", np64(out["dX"]), dX, off)
    for p in range(len(ins)):
        errs.update(block_errors(f"Y{p}", np64(out["Y"][p]), fw[p][0], off))
        for k in range(len(ins[p].ranks)):
            errs[f"dA{p}.{k}"] = relerr(np64(out["dA"][p][k]), dA[p][k])
            errs[f"dB{p}.{k}"] = relerr(np64(out["dB"][p][k]), dB[p][k])
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"{label}: relative Frobenius error above {tol}: {bad}"
    return errs


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", [
    # T, h, [d_p], tokens, [ranks per projection], lead
    (300, 72, [136, 40, 72], [100, 0, 57, 130], [[4, 8, 1, 24], [2, 2, 2, 2], [16, 1, 8, 3]], 5),   # generic kernels
    (513, 200, [264, 264], [513], [[16], [8]], 0),                                                     # two projections, one task
    (257, 64, [64, 128], [], [[], []], 0),                                                             # no adapters
    (1000, 192, [320, 64, 128], [100, 0, 333, 500], [[8, 24, 128, 64], [16, 16, 16, 16], [64, 8, 8, 32]], 7),  # MFMA in bf16
    (1537, 448, [576, 192, 192, 64], [1, 255, 257, 1024], [[64, 32, 8, 16]] * 4, 0),                   # four projections
    (640, 256, [256], [320, 320], [[16, 32]], 0),                                                      # a group of one
    (17000, 128, [128, 64], [9000, 0, 7990], [[16, 8, 64], [32, 32, 8]], 3),                           # 64-row tiles in the shared pass
    (900, 128, [192, 64], [130, 700], [[128, 8], [64, 128]], 3),                                       # two projections, rank 128
    (777, 320, [64, 64, 128, 64], [300, 77, 400], [[8, 32, 16], [32, 8, 8], [16, 16, 16], [24, 8, 32]], 0),  # four, ranks <= 32
])
def test_group_small_shapes(dtype, case):
    T, h, ds, tokens, rk, lead = case
    ins = _group_inputs(T, h, ds, tokens, rk, dtype, lead=lead, seed=23)
    out = run_group(ins)
    check_group(ins, out, TOL[dtype], label=f"group {case}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", [
    (1300, 256, [384, 128, 64], [1, 300, 211, 512, 40], [[8, 128, 8, 64, 16], [64, 8, 16, 8, 32], [8, 8, 64, 16, 8]], 100),
    (700, 320, [192, 64, 128], [31, 33, 95, 97, 160, 161], [[8, 16, 8, 16, 8, 16]] * 3, 17),
])
def test_group_lora_terms_alone(dtype, case):
    """Groups of three with every W_p = 0: each Y_p and the summed dX are the LoRA terms alone,
    held to the tolerance task by task."""
    T, h, ds, tokens, rk, lead = case
    ins = _group_inputs(T, h, ds, tokens, rk, dtype, lead=lead, seed=27)
    for i in ins:
        i.W.zero_()
    out = run_group(ins)
    check_group(ins, out, TOL[dtype], label=f"group W=0 {case}")


def test_group_matches_single_calls():
    """Each projection's Y and dB_k are bit-identical to the single-projection entry points, dA_k
    up to the order of fp32 additions; dX agrees with the sum of the single calls' dX up to
    their bf16 roundings."""
    from tests.parity_util import run_hip
    ins = _group_inputs(1024, 256, [384, 128], [300, 724], [[16, 32], [8, 64]], torch.bfloat16, seed=29)
    out = run_group(ins)
    total = None
    for p, i in enumerate(ins):
        one = run_hip(i)
        assert torch.equal(one["Y"], out["Y"][p])
        for k in range(2):
            assert torch.equal(one["dB"][k], out["dB"][p][k])
            # dA: the same products in fp32; the single call may add them in another order
            # (it splits a task's tokens over blocks when few blocks would run)
            assert relerr(np64(one["dA"][k]), np64(out["dA"][p][k])) <= 1e-5
        total = np64(one["dX"]) if total is None else total + np64(one["dX"])
    assert relerr(np64(out["dX"]), total) <= 1e-2


def test_group_accumulate_and_skip_dx():
    ins = _group_inputs(384, 128, [192, 64], [128, 0, 200], [[8, 16, 16], [8, 8, 8]], torch.bfloat16, lead=16, seed=3)
    base = run_group(ins)
    acc = run_group(ins, accumulate=True, want_dx=False, preset=(0.5, -1.5))
    assert acc["dX"] is None
    for p in range(2):
        for k in range(3):
            assert relerr(np64(acc["dA"][p][k]), np64(base["dA"][p][k]) + 0.5) <= 1e-6
            assert relerr(np64(acc["dB"][p][k]), np64(base["dB"][p][k]) - 1.5) <= 1e-6
        assert not base["dA"][p][1].any() and not base["dB"][p][1].any()


@pytest.mark.parametrize("path", [1, 2, 3])
def test_group_kernel_paths_agree(path):
    from paper_2312_02515_amd import binding as mb
    ins = _group_inputs(777, 256, [384, 128, 64], [300, 77, 400], [[16, 64, 8], [8, 8, 8], [32, 16, 8]], torch.bfloat16,
                        seed=13)
    old = mb.set_kernel_path(path)
    try:
        out = run_group(ins)
    finally:
        mb.set_kernel_path(old)
    check_group(ins, out, TOL[torch.bfloat16], label=f"group path{path}")


def test_group_llama2_13b_qkv_sampled():
    """q, k, v of the Llama-2-13B layer configuration at full size (T = 32768, 5120 -> 5120 x 3,
    16 adapters of ranks {8,16,32,64}): sampled complete rows of every Y_p and of the summed dX,
    whole dA_pk, dB_pk for three adapters of each projection."""
    w = wl.WORKLOADS["llama2_13b_layer"]
    ins = [wl.make_workload_inputs(w, p, device=DEV, seed=0) for p in range(3)]
    for i in ins[1:]:
        i.X = ins[0].X
    out = run_group(ins, poison=False)
    rows = wl.sample_rows(ins[0].seg_offsets, w.T, per_adapter=3, seed=5)
    rs, off2 = orc.gather_rows_problem(rows, ins[0].seg_offsets, w.T)
    idx = torch.as_tensor(rs, device=DEV)
    Xs = np64(ins[0].X[idx])
    Ws = [np64(i.W) for i in ins]
    As = [[np64(a) for a in i.A] for i in ins]
    Bs = [[np64(b) for b in i.B] for i in ins]
    ss = [i.scalings for i in ins]
    fw = orc.group_forward(Xs, Ws, off2, As, Bs, ss)
    dXr, _, _ = orc.group_backward(Xs, Ws, [np64(i.dY[idx]) for i in ins], off2, As, Bs, ss)
    tol = TOL[torch.bfloat16]
    errs = row_errors("dX", np64(out["dX"][idx]), dXr, rs)
    for p in range(3):
        errs.update(row_errors(f"Y{p}", np64(out["Y"][p][idx]), fw[p][0], rs))
        for k in (1, 6, 15):
            lo, hi = ins[p].seg_offsets[k], ins[p].seg_offsets[k + 1]
            ga, gb = orc.adapter_gradients(np64(ins[0].X[lo:hi]), np64(ins[p].dY[lo:hi]), As[p][k], Bs[p][k], ss[p][k])
            errs[f"dA{p}.{k}"] = relerr(np64(out["dA"][p][k]), ga)
            errs[f"dB{p}.{k}"] = relerr(np64(out["dB"][p][k]), gb)
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"qkv group: {bad}"
    assert torch.isfinite(out["dX"]).all()
