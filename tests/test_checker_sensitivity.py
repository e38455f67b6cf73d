"""CPU-only tests of the parity checkers themselves (tests/parity_util.py).

The GPU tests are only as sharp as their checker.  Here the checker is fed "outputs" built
from the oracle with one mistake planted (on the CPU, in a copy of the oracle's result): a
single adapter's LoRA term of Eq. "forward" or Eq. "grad_output" removed or mis-scaled, one
gradient dropped, one row block shifted.  Every such output must be rejected; the oracle's
own result, rounded to the storage type like a kernel would, must be accepted.
"""
import numpy as np
import pytest
import torch

from paper_2312_02515_amd import workloads as wl
from tests.parity_util import (LORA_TERM_CASES, MFMA_SMALL_CASES, TOL, check_full, check_sampled, np64, oracle_full,
                               row_blocks, zero_base_weight)


def _inputs(case, dtype, seed, zero_w=False):
    T, h, d, tokens, ranks, lead = case
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    scal = [0.5 + 0.25 * i for i in range(len(ranks))]
    inp = wl.make_inputs(T, h, d, off, ranks, scal, dtype, device="cpu", seed=seed, sigma_w=1.0 / np.sqrt(h))
    return zero_base_weight(inp) if zero_w else inp


def _as_output(ref, dtype):
    """What a correct kernel would return: the oracle's values rounded to the storage type."""
    return {"Y": torch.from_numpy(ref["Y"]).to(dtype), "dX": torch.from_numpy(ref["dX"]).to(dtype),
            "dA": [torch.from_numpy(a).to(torch.float32) for a in ref["dA"]],
            "dB": [torch.from_numpy(b).to(torch.float32) for b in ref["dB"]]}


def _lora_terms(inp, k):
    """Adapter k's terms s_k x_k A_k B_k and s_k dy_k B_k^T A_k^T, for planting mistakes."""
    lo, hi = inp.seg_offsets[k], inp.seg_offsets[k + 1]
    A, B, s = np64(inp.A[k]), np64(inp.B[k]), inp.scalings[k]
    ly = s * (np64(inp.X[lo:hi]) @ A) @ B
    lx = s * (np64(inp.dY[lo:hi]) @ B.T) @ A.T
    return lo, hi, ly, lx


@pytest.mark.parametrize("zero_w", [False, True])
@pytest.mark.parametrize("case", LORA_TERM_CASES)
def test_checker_accepts_the_rounded_oracle(case, zero_w):
    inp = _inputs(case, torch.bfloat16, 11, zero_w)
    ref = oracle_full(inp)
    check_full(inp, _as_output(ref, torch.bfloat16), TOL[torch.bfloat16], ref=ref)


@pytest.mark.parametrize("case", MFMA_SMALL_CASES)
def test_checker_rejects_a_missing_lora_term(case):
    """The shapes and inputs of the GPU tests' MFMA cases: removing any one adapter's term from
    Y, or from dX, must fail.  With W = 0 always; with the tests' own W whenever the term weighs
    more than the tolerance within its own task's rows (one norm over the whole tensor used to
    let every one of them pass) -- a term below the tolerance of its block is what the W = 0
    cases are for."""
    tol = TOL[torch.bfloat16]
    caught_with_w = 0
    for zero_w in (False, True):
        inp = _inputs(case, torch.bfloat16, 11, zero_w)
        ref = oracle_full(inp)
        for k in range(len(inp.ranks)):
            lo, hi, ly, lx = _lora_terms(inp, k)
            if hi == lo:
                continue
            for name, term in (("Y", ly), ("dX", lx)):
                weight = np.linalg.norm(term) / np.linalg.norm(ref[name][lo:hi])
                if not zero_w and weight < 1.5 * tol:
                    continue
                caught_with_w += not zero_w
                wrong = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in ref.items()}
                wrong[name][lo:hi] -= term
                with pytest.raises(AssertionError, match=rf"{name}\[task{k}\]"):
                    check_full(inp, _as_output(wrong, torch.bfloat16), tol, ref=ref)
    if case == MFMA_SMALL_CASES[2]:
        assert caught_with_w >= 4  # here most terms are visible even beside the base term


@pytest.mark.parametrize("case", LORA_TERM_CASES)
def test_checker_rejects_a_mis_scaled_lora_term(case):
    """With W = 0 the tolerance applies to the LoRA term itself: a term off by 5 % fails."""
    inp = _inputs(case, torch.bfloat16, 19, zero_w=True)
    ref = oracle_full(inp)
    for k in range(len(inp.ranks)):
        lo, hi, ly, lx = _lora_terms(inp, k)
        if hi == lo:
            continue
        for name, term in (("Y", ly), ("dX", lx)):
            wrong = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in ref.items()}
            wrong[name][lo:hi] -= 0.05 * term
            with pytest.raises(AssertionError, match=rf"{name}\[task{k}\]"):
                check_full(inp, _as_output(wrong, torch.bfloat16), TOL[torch.bfloat16], ref=ref)


def test_checker_rejects_leaks_into_rows_of_no_task():
    """Rows before the first and after the last task hold the base term only; with W = 0 they
    must be exact zeros, so anything leaking there fails."""
    inp = _inputs(LORA_TERM_CASES[3], torch.bfloat16, 5, zero_w=True)
    ref = oracle_full(inp)
    names = [b[0] for b in row_blocks(inp.seg_offsets, inp.X.shape[0])]
    assert names[0] == "lead" and names[-1] == "tail"
    for row, blk in ((0, "lead"), (inp.X.shape[0] - 1, "tail")):
        wrong = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in ref.items()}
        wrong["Y"][row, 3] = 0.1
        with pytest.raises(AssertionError, match=rf"Y\[{blk}\]"):
            check_full(inp, _as_output(wrong, torch.bfloat16), TOL[torch.bfloat16], ref=ref)


def test_checker_rejects_wrong_gradients():
    inp = _inputs(MFMA_SMALL_CASES[2], torch.bfloat16, 7)
    ref = oracle_full(inp)
    for k in range(len(inp.ranks)):
        for name in ("dA", "dB"):
            wrong = {"Y": ref["Y"], "dX": ref["dX"], "dA": [a.copy() for a in ref["dA"]], "dB": [b.copy() for b in ref["dB"]]}
            wrong[name][k] *= 1.05   # e.g. a scaling applied twice or dropped
            with pytest.raises(AssertionError, match=f"{name}{k}"):
                check_full(inp, _as_output(wrong, torch.bfloat16), TOL[torch.bfloat16], ref=ref)


def test_sampled_checker_holds_every_row_to_the_tolerance():
    """The row-sampled checker used at the benchmark's sizes: one wrong row among hundreds
    fails even though a norm over all sampled rows would hide it."""
    case = (4096, 256, 320, [1000, 24, 2000, 1000], [8, 16, 32, 64], 40)
    inp = _inputs(case, torch.bfloat16, 3)
    ref = oracle_full(inp)
    T = inp.X.shape[0]
    rows = wl.sample_rows(inp.seg_offsets, T, per_adapter=4, seed=1)
    # every 256-row tile is represented, with its first and last row
    tiles = {r // 256 for r in rows}
    assert tiles == set(range((T + 255) // 256))
    assert all(t * 256 in rows and min(T, (t + 1) * 256) - 1 in rows for t in tiles)
    good = _as_output(ref, torch.bfloat16)
    check_sampled(inp, good, TOL[torch.bfloat16], rows)
    victim = rows[len(rows) // 2]
    for name in ("Y", "dX"):
        bad = {n: (v.clone() if torch.is_tensor(v) else v) for n, v in good.items()}
        bad[name][victim] *= 1.06
        with pytest.raises(AssertionError, match=rf"{name}\[worst row {victim}\]"):
            check_sampled(inp, bad, TOL[torch.bfloat16], rows)
