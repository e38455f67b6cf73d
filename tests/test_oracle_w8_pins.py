"""Pins for the oracle of the 8-bit frozen base weight (oracle/w8_oracle.py): each check holds
it against something that is not its own code path -- a hand-derived example, weights on the
code's grid (exact recovery, and through it the already pinned plain operator), exact rational
arithmetic, invariants of an absmax code, and a scalar evaluation of the dequantised product."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import batchlora_oracle as orc
from oracle import w8_oracle as w8

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _weights(rng, h, d, spread=True):
    """fp32 weights whose columns have very different magnitudes (a per-column code must follow
    them; a per-row or per-tensor code cannot)."""
    W = rng.standard_normal((h, d)).astype(np.float32)
    if spread:
        W *= (2.0 ** rng.integers(-8, 5, size=d)).astype(np.float32)[None, :]
    return W


def _grid_weights(rng, h, d):
    """Weights that lie on the code's grid: W[i, j] = k_ij g_j, integer |k_ij| <= 127 with
    max_i |k_ij| = 127, g_j a power of two (different per column, so that c_j = g_j exactly)."""
    k = rng.integers(-127, 128, size=(h, d))
    k[rng.integers(0, h, size=d), np.arange(d)] = 127 * rng.choice([-1, 1], size=d)
    g = 2.0 ** rng.integers(-9, 3, size=d)
    return (k * g[None, :]).astype(np.float32), k.astype(np.int8), g.astype(np.float32)


def test_hand_derived_example():
    with open(os.path.join(GOLDEN, "w8_worked_example.json")) as f:
        g = json.load(f)
    Wq, c = w8.quantize_w8(np.array(g["W"], np.float32))
    assert Wq.dtype == np.int8 and c.dtype == np.float32
    assert np.array_equal(Wq, np.array(g["Wq"], np.int8))
    assert np.array_equal(c, np.array(g["c"], np.float32))
    assert np.array_equal(w8.dequantize_w8(Wq, c), np.array(g["W_hat"], np.float64))
    for mode in ("bf16", "f32"):   # every W^ of the example has at most 7 significant bits
        assert np.array_equal(w8.dequantize_w8_storage(Wq, c, mode), np.array(g["W_hat"], np.float32))
    H, Z = w8.forward_w8(g["X"], Wq, c, [0], [], [], [])
    dX, dA, dB = w8.backward_w8(g["X"], Wq, c, g["dH"], [0], [], [], [])
    assert Z == [] and dA == [] and dB == []
    assert np.array_equal(H, np.array(g["H"], np.float64))
    assert np.array_equal(dX, np.array(g["dX"], np.float64))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_weights_on_the_grid_are_recovered_exactly(seed):
    """Closed form: a column k_ij g_j with max |k_ij| = 127 has c_j = g_j and code k_ij; the
    dequantised weight is the weight.  Columns differ in g_j by factors up to 2^11 and the
    matrix is not square, so a scale taken per row, per tensor or from the wrong axis fails."""
    rng = np.random.default_rng(seed)
    W, k, g = _grid_weights(rng, 37, 11)
    Wq, c = w8.quantize_w8(W)
    assert np.array_equal(Wq, k)
    assert np.array_equal(c, g)
    assert np.array_equal(w8.dequantize_w8(Wq, c), W.astype(np.float64))
    assert np.array_equal(w8.dequantize_w8_storage(Wq, c, "f32"), W)


@pytest.mark.parametrize("seed", [3, 4])
def test_operator_on_grid_weights_is_the_plain_operator(seed):
    """With W on the grid W^ = W, so forward_w8 / backward_w8 must return exactly what the plain
    operator (pinned in test_oracle_pins.py) returns for W -- LoRA terms, split positions,
    uncovered rows and all."""
    rng = np.random.default_rng(seed)
    T, h, d = 23, 12, 7
    W, k, g = _grid_weights(rng, h, d)
    off = [2, 9, 9, 20]
    ranks = [2, 3, 1]
    X = rng.standard_normal((T, h))
    dH = rng.standard_normal((T, d))
    A = [rng.standard_normal((h, r)) for r in ranks]
    B = [rng.standard_normal((r, d)) for r in ranks]
    s = [0.5, 2.0, 1.25]
    Wq, c = w8.quantize_w8(W)
    H, Z = w8.forward_w8(X, Wq, c, off, A, B, s)
    H0, Z0 = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = w8.backward_w8(X, Wq, c, dH, off, A, B, s)
    dX0, dA0, dB0 = orc.backward(X, W, dH, off, A, B, s)
    assert np.array_equal(H, H0) and np.array_equal(dX, dX0)
    for i in range(3):
        assert np.array_equal(Z[i], Z0[i]) and np.array_equal(dA[i], dA0[i]) and np.array_equal(dB[i], dB0[i])


@pytest.mark.parametrize("seed", [5, 6])
def test_half_step_bound_in_exact_arithmetic(seed):
    """Against exact rationals: c_j is absmax_j / 127 to within fp32 rounding, every code is a
    nearest integer of W / c_j (to within the rounding of one fp32 division), the largest
    element of a column gets +-127, and |W^ - W| <= c_j / 2."""
    rng = np.random.default_rng(seed)
    W = _weights(rng, 29, 6)
    Wq, c = w8.quantize_w8(W)
    for j in range(W.shape[1]):
        col = [Fraction(float(v)) for v in W[:, j]]
        absmax = max(abs(v) for v in col)
        cj = Fraction(float(c[j]))
        assert abs(cj - absmax / 127) <= absmax / 127 * Fraction(1, 2 ** 23)
        for i, v in enumerate(col):
            q = int(Wq[i, j])
            ratio = v / cj
            assert abs(ratio - q) <= Fraction(1, 2) + abs(ratio) * Fraction(1, 2 ** 22)
            assert abs(q * cj - v) <= cj / 2 * (1 + Fraction(1, 2 ** 15))
            if abs(v) == absmax:
                assert abs(q) == 127 and (q > 0) == (v > 0)
    assert np.all(np.abs(Wq.astype(int)) <= 127)


def test_antisymmetry_rescaling_and_zero_column():
    rng = np.random.default_rng(7)
    W = _weights(rng, 31, 9)
    W[:, 4] = 0.0
    Wq, c = w8.quantize_w8(W)
    # all-zero column: code 0, scale 0, dequantised 0 (no NaN from 0 / 0)
    assert c[4] == 0 and not Wq[:, 4].any()
    assert np.array_equal(w8.dequantize_w8(Wq, c)[:, 4], np.zeros(31))
    assert np.all(np.isfinite(w8.dequantize_w8(Wq, c)))
    # -W has the negated codes and the same scales (rint is odd, halves to even on both sides)
    Wq_n, c_n = w8.quantize_w8(-W)
    assert np.array_equal(Wq_n, -Wq) and np.array_equal(c_n, c)
    # a power-of-two factor per column moves into the scale and leaves the codes alone
    f = (2.0 ** rng.integers(-6, 7, size=9)).astype(np.float32)
    Wq_s, c_s = w8.quantize_w8(W * f[None, :])
    assert np.array_equal(Wq_s, Wq) and np.array_equal(c_s, c * f)
    # permuting the rows permutes the codes; permuting columns permutes codes and scales
    pr, pc = rng.permutation(31), rng.permutation(9)
    Wq_p, c_p = w8.quantize_w8(W[pr][:, pc])
    assert np.array_equal(Wq_p, Wq[pr][:, pc]) and np.array_equal(c_p, c[pc])


def test_storage_rounding():
    """dequantize_w8_storage: fp32 product, then nearest-even bfloat16.  Checked against the
    defining property of round-to-nearest on 8-bit significands: the result has at most 8
    significant bits, is within half a unit in the last place of the fp32 product, and ties
    (products whose dropped 16 bits are exactly 0x8000) go to the even neighbour."""
    rng = np.random.default_rng(8)
    Wq = rng.integers(-127, 128, size=(64, 40)).astype(np.int8)
    c = (rng.uniform(0.5, 1.0, size=40) * 2.0 ** rng.integers(-10, 0, size=40)).astype(np.float32)
    c[0] = np.float32(1.0 + 2.0 ** -7)          # 3 * c = 3.0234375 = 1.1000001 1000...b: a tie in bf16
    Wq[0, 0] = 3
    prod = Wq.astype(np.float32) * c[None, :]
    assert np.array_equal(w8.dequantize_w8_storage(Wq, c, "f32"), prod)
    got = w8.dequantize_w8_storage(Wq, c, "bf16")
    assert got.dtype == np.float32
    bits = got.view(np.uint32)
    assert not (bits & 0xFFFF).any()                       # representable in bfloat16
    nz = prod != 0
    ulp = 2.0 ** (np.floor(np.log2(np.abs(prod[nz]))) - 7)  # spacing of bfloat16 at that magnitude
    assert np.all(np.abs(got[nz].astype(np.float64) - prod[nz]) <= ulp / 2)
    assert np.array_equal(got[~nz], prod[~nz])
    # the planted tie: 3.0234375 lies halfway between 3.015625 (odd last bit) and 3.03125 (even)
    assert prod[0, 0] == np.float32(3.0234375) and got[0, 0] == np.float32(3.03125)
    # -tie rounds to the negated value
    Wq[0, 0] = -3
    assert w8.dequantize_w8_storage(Wq, c, "bf16")[0, 0] == np.float32(-3.03125)


def test_base_product_by_scalar_evaluation():
    """The dequantised base product element by element in plain Python floats:
    H[i, j] = c_j sum_l X[i, l] Wq[l, j]  and  dX[i, l] = sum_j dH[i, j] c_j Wq[l, j]
    (the scale of an OUTPUT feature multiplies that feature's column of H and that feature's
    term of the input gradient)."""
    rng = np.random.default_rng(9)
    T, h, d = 5, 6, 4
    W = _weights(rng, h, d)
    Wq, c = w8.quantize_w8(W)
    X = rng.integers(-3, 4, size=(T, h)).astype(np.float64)
    dH = rng.integers(-3, 4, size=(T, d)).astype(np.float64)
    H, _ = w8.forward_w8(X, Wq, c, [0], [], [], [])
    dX, _, _ = w8.backward_w8(X, Wq, c, dH, [0], [], [], [])
    for i in range(T):
        for j in range(d):
            acc = 0
            for l in range(h):
                acc += int(X[i, l]) * int(Wq[l, j])
            assert H[i, j] == pytest.approx(float(c[j]) * acc, rel=1e-13, abs=1e-300)
        for l in range(h):
            acc = 0.0
            for j in range(d):
                acc += float(dH[i, j]) * float(c[j]) * int(Wq[l, j])
            assert dX[i, l] == pytest.approx(acc, rel=1e-12, abs=1e-12)


def test_code_error_is_what_the_operator_sees():
    """forward_w8 differs from the plain forward on W by exactly X (W^ - W): the adapters' terms
    and gradients are untouched by the code (Eq. "grad_lora" does not contain W)."""
    rng = np.random.default_rng(10)
    T, h, d = 17, 10, 6
    W = _weights(rng, h, d, spread=False)
    off, ranks, s = [0, 8, 17], [2, 4], [1.0, 0.5]
    X = rng.standard_normal((T, h))
    dH = rng.standard_normal((T, d))
    A = [rng.standard_normal((h, r)) for r in ranks]
    B = [rng.standard_normal((r, d)) for r in ranks]
    Wq, c = w8.quantize_w8(W)
    E = w8.dequantize_w8(Wq, c) - W.astype(np.float64)
    assert 0 < np.abs(E).max() <= float(c.max()) / 2 * (1 + 1e-6)
    H, Z = w8.forward_w8(X, Wq, c, off, A, B, s)
    H0, Z0 = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = w8.backward_w8(X, Wq, c, dH, off, A, B, s)
    dX0, dA0, dB0 = orc.backward(X, W, dH, off, A, B, s)
    assert np.allclose(H - H0, X @ E, rtol=0, atol=1e-12)
    assert np.allclose(dX - dX0, dH @ E.T, rtol=0, atol=1e-12)
    for k in range(2):
        assert np.array_equal(Z[k], Z0[k]) and np.array_equal(dA[k], dA0[k]) and np.array_equal(dB[k], dB0[k])
