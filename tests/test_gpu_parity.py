"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle
on the same seeded inputs.  Tolerance: relative Frobenius error per output tensor
(Y, dX, every dA_k, every dB_k) <= 2e-2 in bf16 mode and <= 1e-5 in fp32 mode."""
import numpy as np
import pytest
import torch

from paper_2312_02515_amd import workloads as wl
from tests.parity_util import (LORA_TERM_CASES, MFMA_SMALL_CASES, TOL, check_full, check_sampled, np64, relerr,
                               run_hip, zero_base_weight)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(T, h, d, tokens, ranks, dtype, lead=0, seed=0, scal=None):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    assert off[-1] <= T
    s = scal if scal is not None else [2.0] * len(ranks)
    return wl.make_inputs(T, h, d, off, ranks, s, dtype, device=DEV, seed=seed, sigma_w=1.0 / np.sqrt(h))


def test_tiny_f32_workload():
    """Configuration 1 of the benchmark description, fp32 mode."""
    w = wl.WORKLOADS["tiny_f32"]
    inp = wl.make_workload_inputs(w, 0, device=DEV, seed=0)
    out = run_hip(inp)
    check_full(inp, out, TOL[torch.float32], label="tiny_f32")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", [
    # T, h, d, tokens, ranks, lead
    (0 + 300, 72, 136, [100, 0, 57, 130], [4, 8, 1, 24], 5),       # ragged, empty segment, uncovered rows
    (513, 200, 264, [513], [16], 0),                                  # one adapter, ragged tail
    (257, 64, 64, [], [], 0),                                         # no adapters: plain linear
    (640, 256, 320, [64, 192, 128, 256], [8, 16, 32, 64], 0),         # tile-aligned mixed ranks
    (700, 328, 264, [1, 63, 65, 300, 200], [64, 3, 128, 17, 40], 30),  # odd everything, rank up to 128
] + MFMA_SMALL_CASES)  # and the shapes the MFMA kernels take, ragged in every other way
def test_small_shapes(dtype, case):
    T, h, d, tokens, ranks, lead = case
    inp = _inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=11, scal=[0.5 + 0.25 * i for i in range(len(ranks))])
    out = run_hip(inp)
    check_full(inp, out, TOL[dtype], label=f"{case}")


@pytest.mark.parametrize("case", [
    # T, h, d, tokens, ranks, lead -- contraction tiles of 64 (base + LoRA) forward / backward:
    (300, 64, 64, [], [], 0),               # 1 / 1   no adapter, one tile: nothing to prefetch
    (300, 64, 128, [300], [8], 0),          # 2 / 3   one base tile and one LoRA tile
    (300, 128, 64, [100, 150], [64, 16], 20),  # 3-4 / 2-3  two tasks in one row tile
    (300, 64, 64, [300], [128], 0),         # 3 / 3   rank 128: two LoRA tiles behind one base tile
    (520, 192, 128, [260, 260], [32, 128], 0),  # 4-5 / 3-4, two row tiles
    (300, 256, 192, [200], [16], 50),       # 5 / 4   just below the depth where the loop proper starts
])
def test_short_contractions(case):
    """The base-product kernel keeps three tiles of A and two of the weight in flight; with
    fewer tiles than that in all (small h or d, with and without LoRA tiles behind them) its
    prologue and its last tiles take their short forms."""
    T, h, d, tokens, ranks, lead = case
    inp = _inputs(T, h, d, tokens, ranks, torch.bfloat16, lead=lead, seed=23, scal=[1.0 + 0.5 * i for i in range(len(ranks))])
    out = run_hip(inp)
    check_full(inp, out, TOL[torch.bfloat16], label=f"short {case}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", LORA_TERM_CASES)
def test_lora_term_alone(dtype, case):
    """W = 0: every task's rows of Y and dX are the LoRA terms of Eq. "forward" and
    Eq. "grad_output" alone, so the tolerance applies to those terms directly, task by task
    (bf16: the terms folded into the MFMA base-product kernel as extra contraction tiles);
    rows of no task must come out as exact zeros."""
    T, h, d, tokens, ranks, lead = case
    inp = zero_base_weight(_inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=19,
                                   scal=[0.5 + 0.25 * i for i in range(len(ranks))]))
    out = run_hip(inp)
    check_full(inp, out, TOL[dtype], label=f"W=0 {case}")
    off = inp.seg_offsets
    assert not out["Y"][:off[0]].any() and not out["Y"][off[-1]:].any()
    assert not out["dX"][:off[0]].any() and not out["dX"][off[-1]:].any()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_accumulate_and_skip_dx(dtype):
    inp = _inputs(384, 128, 192, [128, 0, 200], [8, 4, 16], dtype, lead=16, seed=3)
    base = run_hip(inp)
    pre_a = [torch.full_like(t, 0.5) for t in base["dA"]]
    pre_b = [torch.full_like(t, -1.5) for t in base["dB"]]
    acc = run_hip(inp, accumulate=True, want_dx=False, preset_grads=(pre_a, pre_b))
    assert acc["dX"] is None
    for k in range(3):
        ea = relerr(np64(acc["dA"][k]), np64(base["dA"][k]) + 0.5)
        eb = relerr(np64(acc["dB"][k]), np64(base["dB"][k]) - 1.5)
        assert ea <= 1e-6 and eb <= 1e-6
    # empty segment: overwrite mode gave zeros, accumulate mode left the preset
    assert not base["dA"][1].any() and not base["dB"][1].any()
    assert torch.equal(acc["dA"][1], pre_a[1]) and torch.equal(acc["dB"][1], pre_b[1])
    assert torch.equal(acc["Y"], base["Y"])


@pytest.mark.parametrize("path", [1, 2, 3])
def test_generic_and_mfma_kernels_agree(path):
    """Every mix of generic and MFMA kernels meets the same tolerance on an MFMA-eligible shape."""
    from paper_2312_02515_amd import binding as mb
    inp = _inputs(777, 256, 384, [300, 77, 400], [16, 64, 8], torch.bfloat16, seed=13)
    old = mb.set_kernel_path(path)
    try:
        out = run_hip(inp)
    finally:
        mb.set_kernel_path(old)
    check_full(inp, out, TOL[torch.bfloat16], label=f"path{path}")


def test_frozen_weight_and_inputs_untouched():
    """W gets no gradient and is never written (section 3.3.1); neither are X, dY, A_k, B_k."""
    inp = _inputs(256, 128, 128, [100, 156], [8, 16], torch.bfloat16, seed=5)
    keep = [t.clone() for t in [inp.W, inp.X, inp.dY] + inp.A + inp.B]
    run_hip(inp)
    for a, b in zip(keep, [inp.W, inp.X, inp.dY] + inp.A + inp.B):
        assert torch.equal(a, b)


def test_deterministic():
    inp = _inputs(1024, 256, 256, [300, 724], [16, 32], torch.bfloat16, seed=9)
    a = run_hip(inp)
    b = run_hip(inp)
    assert torch.equal(a["Y"], b["Y"]) and torch.equal(a["dX"], b["dX"])
    for k in range(2):
        assert torch.equal(a["dA"][k], b["dA"][k]) and torch.equal(a["dB"][k], b["dB"][k])


ISOLATION_CASES = [
    # T, h, d, tokens, ranks, lead, the task that is disturbed
    (768, 256, 256, [256, 256, 256], [8, 16, 8], 0, 1),        # tile-aligned tasks
    (600, 256, 320, [100, 157, 300], [8, 16, 8], 11, 1),       # tasks share 256-row tiles and 32-row fragments
    (1100, 192, 128, [5, 1, 700, 333], [64, 128, 16, 8], 3, 1),  # a one-token task between its neighbours
    (1500, 128, 256, [700, 90, 650], [16, 64, 32], 0, 0),      # the first task; long enough for token-split gradients
]


def _others_identical(a, b, inp, j):
    off = inp.seg_offsets
    K = len(inp.ranks)
    lo, hi = off[j], off[j + 1]
    for name in ("Y", "dX"):
        assert torch.equal(a[name][:lo], b[name][:lo]) and torch.equal(a[name][hi:], b[name][hi:]), name
    for k in range(K):
        if k != j:
            assert torch.equal(a["dA"][k], b["dA"][k]) and torch.equal(a["dB"][k], b["dB"][k]), k


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", ISOLATION_CASES)
def test_isolation_on_gpu(dtype, case):
    """Each adapter uses only its own portion of the data (section 3.3.1): changing task j's
    rows, adapter and scaling leaves every other task's results (and the rows of no task)
    bit-identical, also where tasks share tiles of the kernels."""
    T, h, d, tokens, ranks, lead, j = case
    inp = _inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=21)
    a = run_hip(inp)
    lo, hi = inp.seg_offsets[j], inp.seg_offsets[j + 1]
    inp.X[lo:hi] += 1.0
    inp.dY[lo:hi] *= -2.0
    inp.A[j].mul_(3.0)
    inp.B[j].add_(0.25)
    inp.scalings[j] = 7.0
    b = run_hip(inp)
    _others_identical(a, b, inp, j)
    assert not torch.equal(a["Y"][lo:hi], b["Y"][lo:hi])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("what", ["A", "B", "X", "dY"])
@pytest.mark.parametrize("case", ISOLATION_CASES)
def test_isolation_from_non_finite_values(dtype, what, case):
    """A diverged task (NaN or Inf in its adapter or in its rows) must not leak into its
    neighbours: their Y, dX, dA_k, dB_k stay finite and bit-identical to a clean run."""
    T, h, d, tokens, ranks, lead, j = case
    inp = _inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=22)
    a = run_hip(inp)
    lo, hi = inp.seg_offsets[j], inp.seg_offsets[j + 1]
    bad = {"A": inp.A[j], "B": inp.B[j], "X": inp.X[lo:hi], "dY": inp.dY[lo:hi]}[what]
    flat = bad.view(-1)  # whole tensors and row ranges are contiguous: this writes through
    flat[0::3] = float("nan")
    flat[1::3] = float("inf")
    flat[2::3] = -float("inf")
    b = run_hip(inp)
    _others_identical(a, b, inp, j)
    for name in ("Y", "dX"):
        assert torch.isfinite(b[name][:lo]).all() and torch.isfinite(b[name][hi:]).all()


@pytest.mark.parametrize("K", [1, 4, 64])
def test_batched_equals_separate_calls(K):
    """One batched call over K tasks against K single-task calls of the library on the same
    rows (Listing 2 against Listing 1; the launch-count argument of section 3.3.2 changes the
    number of launches, never the arithmetic): dA_k, dB_k bit-identical, every task's rows of
    Y and dX within the tolerance of each other and of the oracle."""
    from paper_2312_02515_amd import binding as mb
    g = torch.Generator().manual_seed(77 + K)
    tokens = [int(torch.randint(1, 1 + 4096 // K, (1,), generator=g)) for _ in range(K)]
    ranks = [8 * (1 + k % 4) for k in range(K)]
    lead = 5
    T = lead + sum(tokens) + 3
    h, d = 256, 320
    inp = _inputs(T, h, d, tokens, ranks, torch.bfloat16, lead=lead, seed=51, scal=[0.5 + 0.03 * k for k in range(K)])
    batched = run_hip(inp)
    check_full(inp, batched, TOL[torch.bfloat16], label=f"batched K={K}")
    off = inp.seg_offsets
    for k in range(K):
        lo, hi = off[k], off[k + 1]
        one = wl.Inputs(X=inp.X[lo:hi].contiguous(), W=inp.W, dY=inp.dY[lo:hi].contiguous(), A=[inp.A[k]], B=[inp.B[k]],
                        seg_offsets=[0, hi - lo], ranks=[ranks[k]], scalings=[inp.scalings[k]])
        sep = run_hip(one)
        # The separate call runs other launch shapes (few rows: the contraction of s x A is split
        # over waves, a task's tokens over blocks), so fp32 sums may differ in their last bits and
        # a bf16 intermediate in its last place here and there: far inside the tolerance.
        assert relerr(np64(sep["dA"][0]), np64(batched["dA"][k])) <= 1e-3, k
        assert relerr(np64(sep["dB"][0]), np64(batched["dB"][k])) <= 1e-3, k
        assert relerr(np64(sep["Y"]), np64(batched["Y"][lo:hi])) <= 2e-3, k
        assert relerr(np64(sep["dX"]), np64(batched["dX"][lo:hi])) <= 2e-3, k


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_max_adapters(dtype):
    """64 tasks (the library's maximum) of 3..66 tokens with ranks cycling through 8, 16, 24, 32:
    the whole kernel-argument tables are in use."""
    K = 64
    tokens = [3 + k for k in range(K)]
    ranks = [8 * (1 + k % 4) for k in range(K)]
    T = sum(tokens) + 9
    inp = _inputs(T, 128, 192, tokens, ranks, dtype, lead=4, seed=31, scal=[0.5 + 0.05 * k for k in range(K)])
    out = run_hip(inp)
    check_full(inp, out, TOL[dtype], label="64 adapters")


def test_empty_batch_on_gpu():
    """T = 0: both calls return without touching anything; overwrite mode zeroes dA_k, dB_k."""
    from paper_2312_02515_amd import binding as mb
    W = torch.randn(64, 64, device=DEV).to(torch.bfloat16)
    A = [torch.randn(64, 8, device=DEV).to(torch.bfloat16)]
    B = [torch.randn(8, 64, device=DEV).to(torch.bfloat16)]
    prob = mb.Problem(0, 64, 64, W, [0, 0], [8], [2.0], A, B)
    X = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    Y = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    saved, ws = prob.alloc_saved(), prob.alloc_workspace()
    dA, dB = prob.alloc_grads()
    dA[0].fill_(3.0)
    dB[0].fill_(4.0)
    mb.mlora_lora_fwd(prob, X, Y, saved, ws)
    mb.mlora_lora_bwd(prob, X, Y, saved, None, dA, dB, True, ws)
    torch.cuda.synchronize()
    assert (dA[0] == 3.0).all() and (dB[0] == 4.0).all()
    mb.mlora_lora_bwd(prob, X, Y, saved, None, dA, dB, False, ws)
    torch.cuda.synchronize()
    assert not dA[0].any() and not dB[0].any()


@pytest.mark.parametrize("case", [
    (4096, 256, 384, [4096], [32], 0),                 # one task: 16 token ranges per gradient block column
    (2100, 256, 128, [1500, 0, 590], [16, 8, 64], 7),  # ranges that come out empty for the short tasks
    (3000, 128, 640, [700, 2300], [128, 8], 0),        # rank 128, ragged range ends
])
def test_token_split_gradients(case):
    """Few tasks and few columns: the gradient kernels split each task's tokens over blocks and a
    second kernel adds the ranges in order.  Oracle parity, accumulate mode, determinism."""
    T, h, d, tokens, ranks, lead = case
    inp = _inputs(T, h, d, tokens, ranks, torch.bfloat16, lead=lead, seed=37)
    base = run_hip(inp)
    check_full(inp, base, TOL[torch.bfloat16], label=f"token split {case}")
    again = run_hip(inp)
    pre_a = [torch.full_like(t, 0.5) for t in base["dA"]]
    pre_b = [torch.full_like(t, -1.5) for t in base["dB"]]
    acc = run_hip(inp, accumulate=True, preset_grads=(pre_a, pre_b))
    for k in range(len(ranks)):
        assert torch.equal(base["dA"][k], again["dA"][k]) and torch.equal(base["dB"][k], again["dB"][k])
        assert relerr(np64(acc["dA"][k]), np64(base["dA"][k]) + 0.5) <= 1e-6
        assert relerr(np64(acc["dB"][k]), np64(base["dB"][k]) - 1.5) <= 1e-6


def _random_case(seed, mfma):
    """A seeded random problem: K in 0..12 tasks with empty ones, ragged lengths, uncovered rows."""
    g = torch.Generator().manual_seed(1000 + seed)
    ri = lambda lo, hi: int(torch.randint(lo, hi + 1, (1,), generator=g))
    K = ri(0, 12)
    tokens = [0 if ri(0, 5) == 0 else ri(1, 700) for _ in range(K)]
    lead, tail = ri(0, 40), ri(0, 40)
    T = max(lead + sum(tokens) + tail, 1)
    if mfma:
        h, d = 64 * ri(1, 8), 64 * ri(1, 8)
        ranks = [8 * ri(1, 16) for _ in range(K)]
    else:
        h, d = ri(1, 300), ri(1, 300)
        ranks = [ri(1, 128) for _ in range(K)]
    scal = [0.25 * ri(1, 12) for _ in range(K)]
    return T, h, d, tokens, ranks, lead, scal


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_mfma_path(seed):
    T, h, d, tokens, ranks, lead, scal = _random_case(seed, True)
    inp = _inputs(T, h, d, tokens, ranks, torch.bfloat16, lead=lead, seed=seed, scal=scal)
    check_full(inp, run_hip(inp), TOL[torch.bfloat16], label=f"random mfma seed {seed}: {(T, h, d, tokens, ranks, lead)}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("seed", range(4))
def test_random_shapes_generic_path(seed, dtype):
    T, h, d, tokens, ranks, lead, scal = _random_case(100 + seed, False)
    inp = _inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=seed, scal=scal)
    check_full(inp, run_hip(inp), TOL[dtype], label=f"random generic seed {seed}: {(T, h, d, tokens, ranks, lead)}")


def test_hip_graph_capture_and_replay():
    """The entry points allocate nothing and keep all metadata in kernel arguments, so a forward +
    backward pair can be captured into a HIP graph; every replay (with eager work between the
    replays) reproduces the eager result bit for bit, also after the inputs change in place."""
    from paper_2312_02515_amd import binding as mb
    inp = _inputs(1536, 256, 384, [500, 0, 1000], [16, 8, 64], torch.bfloat16, lead=20, seed=41)
    T, h = inp.X.shape
    d = inp.W.shape[1]
    prob = mb.Problem(T, h, d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
    saved, ws = prob.alloc_saved(), prob.alloc_workspace()
    Y = torch.empty((T, d), dtype=torch.bfloat16, device=DEV)
    dX = torch.empty((T, h), dtype=torch.bfloat16, device=DEV)
    dA, dB = prob.alloc_grads()

    def call(stream=None):
        mb.mlora_lora_fwd(prob, inp.X, Y, saved, ws, stream)
        mb.mlora_lora_bwd(prob, inp.X, inp.dY, saved, dX, dA, dB, False, ws, stream)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in [Y, dX] + dA + dB]

    call()
    eager = snapshot()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream())
    for rep in range(3):
        for t in [Y, dX] + dA + dB:
            t.fill_(float("nan"))          # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        for a, b in zip(eager, snapshot()):
            assert torch.equal(a, b), f"replay {rep}"
    # new data in the same buffers: the graph computes on what the buffers hold now
    inp.X.mul_(-0.5)
    inp.dY.add_(0.25)
    call()
    eager2 = snapshot()
    graph.replay()
    for a, b in zip(eager2, snapshot()):
        assert torch.equal(a, b)


def _same_bits(a, b, K):
    assert torch.equal(a["Y"], b["Y"]) and torch.equal(a["dX"], b["dX"])
    for k in range(K):
        assert torch.equal(a["dA"][k], b["dA"][k]) and torch.equal(a["dB"][k], b["dB"][k])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", [
    (300, 72, 136, [100, 0, 57, 130], [4, 8, 1, 24], 5),             # generic kernels, ragged
    (1000, 192, 320, [100, 0, 333, 500], [8, 24, 128, 64], 7),        # MFMA kernels in bf16
    (257, 64, 64, [], [], 0),                                         # no adapters
])
def test_recompute_variant(dtype, case):
    """The activation-recompute entry points (section 4.1: runs with activation checkpointing)
    against the oracle, and bit-identical to the pair that keeps `saved`."""
    T, h, d, tokens, ranks, lead = case
    inp = _inputs(T, h, d, tokens, ranks, dtype, lead=lead, seed=17, scal=[1.5 - 0.25 * i for i in range(len(ranks))])
    out = run_hip(inp, recompute=True)
    check_full(inp, out, TOL[dtype], label=f"recompute {case}")
    _same_bits(out, run_hip(inp), len(ranks))


def test_recompute_variant_accumulate_skip_dx():
    inp = _inputs(384, 128, 192, [128, 0, 200], [8, 16, 16], torch.bfloat16, lead=16, seed=3)
    base = run_hip(inp, recompute=True)
    pre_a = [torch.full_like(t, 0.25) for t in base["dA"]]
    pre_b = [torch.full_like(t, -2.0) for t in base["dB"]]
    acc = run_hip(inp, accumulate=True, want_dx=False, preset_grads=(pre_a, pre_b), recompute=True)
    assert acc["dX"] is None
    for k in range(3):
        assert relerr(np64(acc["dA"][k]), np64(base["dA"][k]) + 0.25) <= 1e-6
        assert relerr(np64(acc["dB"][k]), np64(base["dB"][k]) - 2.0) <= 1e-6


def test_llama2_7b_qproj_full():
    """Configuration 2, every output element against the oracle."""
    w = wl.WORKLOADS["llama2_7b_qproj"]
    inp = wl.make_workload_inputs(w, 0, device=DEV, seed=0)
    out = run_hip(inp, poison=False)
    errs = check_full(inp, out, TOL[torch.bfloat16], label=w.name)
    print(w.name, {k: f"{v:.2e}" for k, v in errs.items()})


def _sampled_workload(name, proj, per_adapter=6, grad_adapters=None):
    w = wl.WORKLOADS[name]
    inp = wl.make_workload_inputs(w, proj, device=DEV, seed=0)
    out = run_hip(inp, poison=False)
    rows = wl.sample_rows(inp.seg_offsets, w.T, per_adapter, seed=proj)
    errs = check_sampled(inp, out, TOL[torch.bfloat16], rows, grad_adapters=grad_adapters,
                         label=f"{name}/{w.projections[proj].name}")
    # properties that hold at any size: every output is finite, W untouched
    assert torch.isfinite(out["Y"]).all() and torch.isfinite(out["dX"]).all()
    print(name, w.projections[proj].name, "max err", f"{max(errs.values()):.2e}")


@pytest.mark.parametrize("proj", [0, 2])
def test_llama2_7b_mlp_sampled(proj):
    """Configuration 3 at full size: sampled complete rows of Y and dX, all dA_k, dB_k."""
    _sampled_workload("llama2_7b_mlp", proj)


def test_llama2_13b_layer_recompute_sampled():
    """Configuration 4, one projection, through the activation-recompute entry points."""
    w = wl.WORKLOADS["llama2_13b_layer"]
    inp = wl.make_workload_inputs(w, 3, device=DEV, seed=0)
    out = run_hip(inp, poison=False, recompute=True)
    rows = wl.sample_rows(inp.seg_offsets, w.T, per_adapter=4, seed=2)
    check_sampled(inp, out, TOL[torch.bfloat16], rows, grad_adapters=[0, 7, 15], label="llama2_13b_layer/o recompute")


@pytest.mark.parametrize("proj", [0, 4, 6])
def test_llama2_13b_layer_sampled(proj):
    """Configuration 4 at full size (q_proj, gate_proj, down_proj shapes), in the launch
    configuration the benchmark times: sampled complete rows of Y and dX, all dA_k, dB_k."""
    _sampled_workload("llama2_13b_layer", proj, per_adapter=4)


@pytest.mark.parametrize("proj", [0, 1])
def test_llama2_70b_mlp_stage_sampled(proj):
    """Configuration 5 at full size: sampled rows, and whole dA_k, dB_k for a seeded third of
    the 32 adapters (each is an independent exact reduction)."""
    picks = [0, 2, 3, 7, 11, 13, 16, 20, 25, 28, 31]
    _sampled_workload("llama2_70b_mlp_stage", proj, per_adapter=2, grad_adapters=picks)
