"""mlora_lora_bwd_static (the backward whose scratch is a fixed array inside the library, for
callers that cannot allocate) against mlora_lora_bwd on the same inputs, through the C ABI:
bit-identical results, on two calls in a row that share the array, the second on a smaller
problem, and a third with other kernels (token-split gradient sums use the scratch as well)."""
import pytest
import torch

from paper_2312_02515_amd import binding as mb
from paper_2312_02515_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(T, h, d, tokens, ranks, dtype, lead, seed):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    return wl.make_inputs(T, h, d, off, ranks, [1.0 + 0.5 * k for k in range(len(ranks))], dtype, device=DEV,
                          seed=seed, sigma_w=h ** -0.5)


def _both(inp):
    T, h = inp.X.shape
    d = inp.W.shape[1]
    prob = mb.Problem(T, h, d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
    assert prob.workspace_bytes() <= mb.MLORA_STATIC_SCRATCH_BYTES
    saved, ws = prob.alloc_saved(), prob.alloc_workspace()
    Y = torch.empty((T, d), dtype=inp.X.dtype, device=DEV)
    mb.mlora_lora_fwd(prob, inp.X, Y, saved, ws)
    outs = []
    for static in (False, True):
        dX = torch.full((T, h), float("nan"), dtype=inp.X.dtype, device=DEV)
        dA, dB = prob.alloc_grads()
        for t in dA + dB:
            t.fill_(float("nan"))
        if static:
            mb.mlora_lora_bwd_static(prob, inp.X, inp.dY, saved, dX, dA, dB, False)
        else:
            ws.fill_(0xFF)
            mb.mlora_lora_bwd(prob, inp.X, inp.dY, saved, dX, dA, dB, False, ws)
        torch.cuda.synchronize()
        outs.append((dX, dA, dB))
    (dX0, dA0, dB0), (dX1, dA1, dB1) = outs
    assert torch.equal(dX0, dX1)
    assert torch.isfinite(dX1).all()
    for a, b in zip(dA0 + dB0, dA1 + dB1):
        assert torch.equal(a, b) and torch.isfinite(b).all()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_backward_matches_workspace_backward(dtype):
    # two calls in a row on the shared array, the second with a smaller input: stale contents of
    # the first call (larger G, wider rows) must not show in the second
    _both(_inputs(3000, 256, 384, [1000, 0, 1500, 400], [64, 8, 128, 16], dtype, 50, seed=61))
    _both(_inputs(700, 128, 192, [300, 77, 200], [8, 16, 8], dtype, 3, seed=62))
    # one long task: its tokens are split over blocks, the partial sums go through the scratch too
    _both(_inputs(4096, 256, 384, [4096], [32], dtype, 0, seed=63))
    _both(_inputs(513, 200, 264, [513], [16], dtype, 0, seed=64))   # generic kernels in both modes


def test_static_scratch_refuses_what_does_not_fit():
    """Sizes beyond the fixed array are refused before any launch."""
    T, h, d = 1 << 18, 64, 64    # G alone: 2^18 rows x 128 ranks x 2 B = 64 MiB
    W = torch.zeros((h, d), dtype=torch.bfloat16, device=DEV)
    A = [torch.zeros((h, 128), dtype=torch.bfloat16, device=DEV)]
    B = [torch.zeros((128, d), dtype=torch.bfloat16, device=DEV)]
    prob = mb.Problem(T, h, d, W, [0, T], [128], [1.0], A, B)
    assert prob.workspace_bytes() > mb.MLORA_STATIC_SCRATCH_BYTES
    dA, dB = prob.alloc_grads()
    with pytest.raises(mb.MloraError) as ei:
        mb.mlora_lora_bwd_static(prob, W, W, W, None, dA, dB, False)   # buffers are never touched
    assert ei.value.status == 6
