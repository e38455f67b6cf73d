"""CPU oracle for the 8-bit frozen base weight of the BatchLoRA operator.

TEST INFRASTRUCTURE ONLY, like batchlora_oracle.py: imported by the tests and by
nothing on the product path; shares no code with the HIP kernels.

The paper's single-GPU setup (section 4.1) keeps the frozen pre-trained weights
in 8 bits to fit its 48 GB cards; it names the technique and gives no format.
The reading taken here (listed with its reasons in this repository's design
notes) is the plain vector-wise absmax code:

  * W [h, d] is coded column by column (one column = one output feature):
        c_j      = max_i |W[i, j]| / 127                      (fp32, one per column)
        Wq[i, j] = rint( W[i, j] / c_j )  in [-127, 127]      (int8; 0 where c_j = 0)
    The code is an integer decided by floating point, so the precision is part of
    the definition: the maximum is exact, the two divisions are IEEE fp32
    divisions, rint rounds halves to even.
  * The weight the operator then uses is  W^[i, j] = Wq[i, j] * c_j.  Only W is
    coded: activations, adapters, gradients and every product stay in the
    operator's own types, and W^ takes the place of W in Eq. "forward" and
    Eq. "grad_output" (the adapters' gradients, Eq. "grad_lora", do not see W).
  * The library hands W^ to its kernels in the storage type: fl32(Wq * c_j)
    rounded to the nearest-even bfloat16 in bf16 mode (`dequantize_w8_storage`);
    this oracle's forward / backward use the exact product in float64.

Not modelled: 8-bit activations, outlier columns kept in 16 bits, any other
code book.  Agreement with the implementation the paper's authors ran is
therefore unpinned ("parity unpinned" for that); what is pinned
(tests/test_oracle_w8_pins.py) is this definition: a hand-derived example in
tests/golden/, exact recovery of weights that lie on the code's grid (which also
ties forward_w8 / backward_w8 to the pinned plain operator), the half-step error
bound against exact rational arithmetic, antisymmetry, invariance under
power-of-two rescaling, an all-zero column, and a scalar brute force of the
dequantised base product.
"""
from __future__ import annotations

import numpy as np

from . import batchlora_oracle as _op

__all__ = [
    "quantize_w8",
    "dequantize_w8",
    "dequantize_w8_storage",
    "forward_w8",
    "backward_w8",
]


def quantize_w8(W):
    """Column-wise absmax code of W [h, d] (values that fp32 holds exactly).

    Returns (Wq int8 [h, d], c float32 [d]).
    """
    W32 = np.ascontiguousarray(np.asarray(W, dtype=np.float32))
    assert W32.ndim == 2
    absmax = np.max(np.abs(W32), axis=0) if W32.shape[0] else np.zeros(W32.shape[1], np.float32)
    c = (absmax / np.float32(127.0)).astype(np.float32)
    Wq = np.zeros(W32.shape, dtype=np.int8)
    for j in range(W32.shape[1]):
        if c[j] > 0:
            code = np.rint(W32[:, j] / c[j])          # fp32 division, halves to even
            Wq[:, j] = np.clip(code, -127, 127).astype(np.int8)
    return Wq, c


def dequantize_w8(Wq, c):
    """W^ = Wq * c_j, exact (an 8-bit integer times an fp32 number fits float64)."""
    Wq = np.asarray(Wq)
    c = np.asarray(c, dtype=np.float32)
    assert Wq.dtype == np.int8 and Wq.ndim == 2 and c.shape == (Wq.shape[1],)
    return Wq.astype(np.float64) * c.astype(np.float64)[None, :]


def _round_to_bf16(x32):
    """fp32 -> nearest-even bfloat16, returned as fp32 (finite inputs)."""
    bits = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    bits = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return bits.view(np.float32)


def dequantize_w8_storage(Wq, c, dtype):
    """W^ as the library stores it for its kernels: the fp32 product fl32(Wq * c_j), and in
    "bf16" mode that product rounded to the nearest-even bfloat16.  Returned as float32."""
    Wq = np.asarray(Wq)
    c = np.asarray(c, dtype=np.float32)
    assert Wq.dtype == np.int8 and c.shape == (Wq.shape[1],)
    prod = Wq.astype(np.float32) * c[None, :]
    if dtype == "bf16":
        return _round_to_bf16(prod)
    assert dtype == "f32"
    return prod


def forward_w8(X, Wq, c, seg_offsets, A, B, s):
    """Eq. "forward" with W^ in the place of W.  Returns (H, Z) as batchlora_oracle.forward."""
    return _op.forward(X, dequantize_w8(Wq, c), seg_offsets, A, B, s)


def backward_w8(X, Wq, c, dH, seg_offsets, A, B, s):
    """Eqs. "grad_lora" and "grad_output" with W^ in the place of W."""
    return _op.backward(X, dequantize_w8(Wq, c), dH, seg_offsets, A, B, s)
