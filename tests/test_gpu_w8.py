"""GPU parity of the 8-bit frozen base weight (section 4.1) through the C ABI: the coder and the
decoder bit for bit against the oracle (integer codes; floating point decides them in fp32 on
both sides), the operator calls against the oracle's forward_w8 / backward_w8 to the operator's
tolerance, and the properties the header promises (bit-identity with the plain calls on the
decoded weight, nothing decoded when dX is not wanted, interchangeable `saved`)."""
import copy

import numpy as np
import pytest
import torch

from oracle import w8_oracle as w8
from paper_2312_02515_amd import workloads as wl
from tests.parity_util import MFMA_SMALL_CASES, TOL, check_full, check_sampled, np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def mb():
    from paper_2312_02515_amd import binding
    assert torch.cuda.is_available()
    return binding


def _spread_columns(W, seed):
    """Seeded power-of-two factor per column, so that the per-column scales really differ."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    f = torch.pow(2.0, torch.randint(-4, 4, (W.shape[1],), generator=g).to(torch.float32)).to(W.device)
    return (W.to(torch.float32) * f[None, :]).to(W.dtype)


def _f32(t):
    return t.detach().to("cpu").to(torch.float32).numpy()


def _case(T, h, d, tokens, ranks, lead, dtype, seed):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    inp = wl.make_inputs(T, h, d, off, ranks, [2.0] * len(ranks), dtype, device=DEV, seed=seed, sigma_w=0.05)
    inp.W = _spread_columns(inp.W, seed)
    return inp


def _run_w8(mb, inp, Wq, c, want_dx=True, accumulate=False):
    T, h = inp.X.shape
    d = Wq.shape[1]
    prob = mb.Problem(T, h, d, None, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B,
                      dtype=inp.X.dtype, device=DEV)
    saved, ws = prob.alloc_saved(), prob.alloc_w8_workspace()
    Y = torch.full((T, d), float("nan"), dtype=inp.X.dtype, device=DEV)
    dX = torch.full((T, h), float("nan"), dtype=inp.X.dtype, device=DEV) if want_dx else None
    dA, dB = prob.alloc_grads()
    for t in dA + dB:
        t.fill_(float("nan"))
    saved.fill_(0xFF)
    ws.fill_(0xFF)
    mb.mlora_lora_fwd_w8(prob, Wq, c, inp.X, Y, saved, ws)
    ws.fill_(0xFF)
    mb.mlora_lora_bwd_w8(prob, Wq, c, inp.X, inp.dY, saved, dX, dA, dB, accumulate, ws)
    torch.cuda.synchronize()
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB, "saved": saved, "ws": ws, "prob": prob}


def _oracle_w8(inp):
    Wq, c = w8.quantize_w8(_f32(inp.W))
    X, dY = np64(inp.X), np64(inp.dY)
    A = [np64(a) for a in inp.A]
    B = [np64(b) for b in inp.B]
    H, _ = w8.forward_w8(X, Wq, c, inp.seg_offsets, A, B, inp.scalings)
    dX, dA, dB = w8.backward_w8(X, Wq, c, dY, inp.seg_offsets, A, B, inp.scalings)
    return {"Y": H, "dX": dX, "dA": dA, "dB": dB}, Wq, c


# ------------------------------------------------------------------ coder / decoder, bit for bit
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("h,d", [(192, 320), (1, 7), (333, 130), (64, 64), (1030, 65), (5, 1)])
def test_quantize_matches_oracle_bit_for_bit(mb, dtype, h, d):
    g = torch.Generator(device="cpu")
    g.manual_seed(h * 1000 + d)
    W = torch.randn((h, d), generator=g).to(dtype)
    W = _spread_columns(W, h + d)
    if d > 3:
        W[:, 2] = 0                                  # all-zero column: scale 0, codes 0
        W[:, 3] = W[0, 3]                            # every element is the maximum
    if h > 4:
        W[1, 0] = -W[:, 0].abs().max()               # the maximum occurs with both signs
        W[2, 0] = W[:, 0].abs().max()
    Wd = W.to(DEV)
    before = Wd.clone()
    Wq, c = mb.mlora_w8_quantize(Wd)
    torch.cuda.synchronize()
    assert torch.equal(Wd, before)
    ref_q, ref_c = w8.quantize_w8(_f32(W))
    assert np.array_equal(c.cpu().numpy(), ref_c), "scales differ"
    assert np.array_equal(Wq.cpu().numpy(), ref_q), "codes differ"


@pytest.mark.parametrize("dtype,mode", [(torch.bfloat16, "bf16"), (torch.float32, "f32")])
@pytest.mark.parametrize("h,d", [(192, 320), (3, 16), (333, 130), (1, 1), (77, 2064)])
def test_dequantize_matches_oracle_bit_for_bit(mb, dtype, mode, h, d):
    """d = 320, 16, 2064 take the 16-codes-per-thread form, 130 and 1 the one-element form."""
    rng = np.random.default_rng(h * 7 + d)
    Wq = rng.integers(-127, 128, size=(h, d)).astype(np.int8)
    c = (rng.uniform(0.5, 1.0, size=d) * 2.0 ** rng.integers(-12, 2, size=d)).astype(np.float32)
    c[0] = 0.0
    got = mb.mlora_w8_dequantize(torch.from_numpy(Wq).to(DEV), torch.from_numpy(c).to(DEV), dtype)
    torch.cuda.synchronize()
    ref = w8.dequantize_w8_storage(Wq, c, mode)
    assert np.array_equal(_f32(got), ref)


# ------------------------------------------------------------------ the operator
W8_CASES = MFMA_SMALL_CASES + [
    (300, 96, 80, [100, 150], [4, 12], 20),          # generic kernels (h, d not multiples of 64)
    (512, 256, 528, [256, 256], [16, 16], 0),        # d a multiple of 16 only
]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("case", range(len(W8_CASES)))
def test_w8_operator_matches_oracle(mb, dtype, case):
    T, h, d, tokens, ranks, lead = W8_CASES[case]
    inp = _case(T, h, d, tokens, ranks, lead, dtype, seed=50 + case)
    ref, ref_q, ref_c = _oracle_w8(inp)
    Wq, c = mb.mlora_w8_quantize(inp.W)
    out = _run_w8(mb, inp, Wq, c)
    assert np.array_equal(Wq.cpu().numpy(), ref_q) and np.array_equal(c.cpu().numpy(), ref_c)
    check_full(inp, out, TOL[dtype], label=f"w8 case {case} {dtype}", ref=ref)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_w8_calls_equal_plain_calls_on_the_decoded_weight(mb, dtype):
    """Bit-identity promised by the header; `saved` is interchangeable; a backward call that
    does not want dX decodes nothing (the head of its workspace stays untouched)."""
    T, h, d, tokens, ranks, lead = MFMA_SMALL_CASES[0]
    inp = _case(T, h, d, tokens, ranks, lead, dtype, seed=77)
    Wq, c = mb.mlora_w8_quantize(inp.W)
    out = _run_w8(mb, inp, Wq, c)
    W_hat = mb.mlora_w8_dequantize(Wq, c, dtype)
    plain = mb.Problem(T, h, d, W_hat, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B)
    saved, ws = plain.alloc_saved(), plain.alloc_workspace()
    Y = torch.empty((T, d), dtype=dtype, device=DEV)
    dX = torch.empty((T, h), dtype=dtype, device=DEV)
    dA, dB = plain.alloc_grads()
    saved.fill_(0xFF)          # as in _run_w8: rows of no task are not written
    mb.mlora_lora_fwd(plain, inp.X, Y, saved, ws)
    mb.mlora_lora_bwd(plain, inp.X, inp.dY, out["saved"], dX, dA, dB, False, ws)   # saved of the w8 forward
    torch.cuda.synchronize()
    assert torch.equal(Y, out["Y"]) and torch.equal(dX, out["dX"])
    assert torch.equal(saved, out["saved"])
    for k in range(len(ranks)):
        assert torch.equal(dA[k], out["dA"][k]) and torch.equal(dB[k], out["dB"][k])
    # dX not wanted: adapter gradients only, no decoding
    prob = out["prob"]
    ws8 = prob.alloc_w8_workspace()
    ws8.fill_(0xA5)
    dA2, dB2 = prob.alloc_grads()
    mb.mlora_lora_bwd_w8(prob, Wq, c, inp.X, inp.dY, saved, None, dA2, dB2, False, ws8)
    torch.cuda.synchronize()
    wbytes = (h * d * W_hat.element_size() + 255) // 256 * 256
    assert bool((ws8[:wbytes] == 0xA5).all())
    for k in range(len(ranks)):
        assert torch.equal(dA2[k], dA[k]) and torch.equal(dB2[k], dB[k])
    # accumulate mode adds to what the buffers hold
    mb.mlora_lora_bwd_w8(prob, Wq, c, inp.X, inp.dY, saved, None, dA2, dB2, True, ws8)
    torch.cuda.synchronize()
    assert torch.equal(dA2[0], dA[0] * 2)


def test_w8_short_workspace_is_refused(mb):
    T, h, d, tokens, ranks, lead = MFMA_SMALL_CASES[1]
    inp = _case(T, h, d, tokens, ranks, lead, torch.bfloat16, seed=3)
    Wq, c = mb.mlora_w8_quantize(inp.W)
    prob = mb.Problem(T, h, d, None, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B,
                      dtype=torch.bfloat16, device=DEV)
    Y = torch.zeros((T, d), dtype=torch.bfloat16, device=DEV)
    short = torch.empty(prob.w8_workspace_bytes() - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(mb.MloraError) as e:
        mb.mlora_lora_fwd_w8(prob, Wq, c, inp.X, Y, prob.alloc_saved(), short)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert not Y.any()


def test_w8_full_size_sampled(mb):
    """q_proj of the Llama-2-13B layer workload at its full size (T = 32768, 5120 x 5120, K = 16),
    in the launch configuration the benchmark's --w8 mode times: complete sampled rows of Y and
    dX, every row held to the tolerance, against the oracle on its own codes; codes and scales of
    the whole weight bit for bit."""
    w = wl.WORKLOADS["llama2_13b_layer"]
    inp = wl.make_workload_inputs(w, 0, device=DEV, seed=0)
    inp.W = _spread_columns(inp.W, 11)
    Wq, c = mb.mlora_w8_quantize(inp.W)
    out = _run_w8(mb, inp, Wq, c)
    ref_q, ref_c = w8.quantize_w8(_f32(inp.W))
    assert np.array_equal(Wq.cpu().numpy(), ref_q) and np.array_equal(c.cpu().numpy(), ref_c)
    p0 = w.projections[0]
    assert mb.Problem(w.T, p0.h, p0.d, inp.W, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B).kernel_path() == 0
    rows = wl.sample_rows(inp.seg_offsets, w.T, per_adapter=2, seed=5, tile=0)
    inp_hat = copy.copy(inp)
    inp_hat.W = w8.dequantize_w8(ref_q, ref_c)        # float64, exact
    check_sampled(inp_hat, out, TOL[torch.bfloat16], rows, grad_adapters=[0, 7, 15], label="w8 q_proj full size")


def test_w8_hip_graph_capture_and_replay(mb):
    """The 8-bit-weight calls allocate nothing either (decoder and operator kernels only, no
    memset): a captured forward + backward pair replays to the eager result bit for bit, with
    eager work between the replays, and follows new codes written into the same buffers."""
    T, h, d, tokens, ranks, lead = MFMA_SMALL_CASES[2]
    inp = _case(T, h, d, tokens, ranks, lead, torch.bfloat16, seed=91)
    Wq, c = mb.mlora_w8_quantize(inp.W)
    prob = mb.Problem(T, h, d, None, inp.seg_offsets, inp.ranks, inp.scalings, inp.A, inp.B,
                      dtype=torch.bfloat16, device=DEV)
    saved, ws = prob.alloc_saved(), prob.alloc_w8_workspace()
    Y = torch.empty((T, d), dtype=torch.bfloat16, device=DEV)
    dX = torch.empty((T, h), dtype=torch.bfloat16, device=DEV)
    dA, dB = prob.alloc_grads()

    def call(stream=None):
        mb.mlora_lora_fwd_w8(prob, Wq, c, inp.X, Y, saved, ws, stream)
        mb.mlora_lora_bwd_w8(prob, Wq, c, inp.X, inp.dY, saved, dX, dA, dB, False, ws, stream)

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
            t.fill_(float("nan"))
        ws.fill_(0x5A)                     # the decoded weight is rebuilt by every call
        torch.cuda.synchronize()
        graph.replay()
        for a, b in zip(eager, snapshot()):
            assert torch.equal(a, b), f"replay {rep}"
    Wq2, c2 = mb.mlora_w8_quantize((inp.W.float() * 1.5).to(torch.bfloat16).flip(0).contiguous())
    Wq.copy_(Wq2)
    c.copy_(c2)
    call()
    eager2 = snapshot()
    graph.replay()
    for a, b in zip(eager2, snapshot()):
        assert torch.equal(a, b)
    assert not torch.equal(eager[0], eager2[0])
