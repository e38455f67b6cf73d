"""CPU fp64 oracle for the BatchLoRA multi-adapter LoRA linear operator.

TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is checked
against; it is imported by the tests, by the smoke check and by the benchmark's
`cpu_baseline` leg, and by nothing on the product path.  It shares no code with
the HIP kernels and imports nothing from the HIP package.

What it computes (paper section 3.3.1, "BatchLoRA Operator"):

  forward   (Eq. "forward"):      H  = X W + rows_k( x_k A_k B_k )
  adapter gradients (Eq. "grad_lora"):
                                  dA_k = x_k^T dh_k B_k^T ,  dB_k = A_k^T x_k^T dh_k
  input gradient (Eq. "grad_output"):
                                  dX = dH W^T + rows_k( dh_k B_k^T A_k^T )
  W is frozen and receives no gradient.

Notation follows the paper: W is [h, d] (input features x output features, as in
Eq. 1 where h = x W), A_k is [h, r_k], B_k is [r_k, d].  X is the row-wise
concatenation of the tasks' token matrices; task k owns rows
[seg_offsets[k], seg_offsets[k+1]).

Readings where the paper is silent (each one is listed with its reason in the
design notes of this repository):
  * LoRA scaling.  The paper's equations carry no alpha/r factor.  Every LoRA
    term here carries one factor s_k (x_k A_k B_k -> s_k x_k A_k B_k), so dA_k,
    dB_k and the LoRA part of dX carry s_k once.  s_k = 1 is the paper verbatim.
  * Rows outside every segment (before seg_offsets[0] or after seg_offsets[K])
    get the base term only.
  * An empty segment yields zero dA_k and dB_k.
  * No bias, no dropout.

Everything is float64.  A matmul (numpy `@`) serves as the library primitive for
each product in the equations; the steps are taken in the order the workflow
paragraph of section 3.3.1 gives them (base product once, split, per-adapter
low-rank products, add back at the split positions), with no blocking or fusion.

Projection groups (group_forward / group_backward): several projections fed by
the same X; their outputs are independent, dX is the sum of their input
gradients.  Pinned by the concatenated-weight identity (the group equals one
projection with W = [W_0 | W_1 | ...], A_k = [A_0k | A_1k | ...] and a
block-diagonal B_k), by a doubled copy of the hand-derived example and by finite
differences of L = sum_p sum(dY_p * Y_p).

Pins (tests/test_oracle_pins.py): a hand-derived integer worked example stored
in tests/golden/, an element-by-element scalar brute force, the merged-weight
closed form of Eq. 1, the B = 0 special case, batched == one-adapter-at-a-time
(Listing 1 vs Listing 2), isolation between tasks, segment permutation,
linearity in s_k, K = 0 reducing to a plain matrix product, and central finite
differences of L = sum(dY * Y).  The paper prints no numeric example, so at
the benchmark sizes the oracle is pinned only through the code that passed
those checks ("parity unpinned" beyond them).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "forward",
    "backward",
    "adapter_gradients",
    "group_forward",
    "group_backward",
    "gather_rows_problem",
    "flops",
]


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _check(X, W, seg_offsets, A, B, s):
    T, h = X.shape
    h2, d = W.shape
    assert h == h2, "X is [T,h], W is [h,d]"
    K = len(A)
    assert len(B) == K and len(s) == K and len(seg_offsets) == K + 1
    prev = 0
    for o in seg_offsets:
        assert 0 <= prev <= o <= T, "segment offsets must be monotone within [0,T]"
        prev = o
    for k in range(K):
        r = A[k].shape[1]
        assert A[k].shape == (h, r) and B[k].shape == (r, d)
    return T, h, d, K


def forward(X, W, seg_offsets, A, B, s):
    """Eq. "forward" with the workflow of section 3.3.1.

    Returns (H, Z) where H is [T,d] and Z[k] = x_k A_k ([t_k, r_k], unscaled) is
    the intermediate a backward pass may reuse.
    """
    X, W = _f64(X), _f64(W)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    T, h, d, K = _check(X, W, seg_offsets, A, B, s)
    # "Y = XW", launched once over the consolidated data
    H = X @ W
    Z = []
    for k in range(K):
        lo, hi = int(seg_offsets[k]), int(seg_offsets[k + 1])
        x_k = X[lo:hi]                      # the split
        z_k = x_k @ A[k]
        L_k = float(s[k]) * (z_k @ B[k])    # L_k = x_k A_k B_k (scaled)
        H[lo:hi] += L_k                     # added back at its original position
        Z.append(z_k)
    return H, Z


def adapter_gradients(x_k, dh_k, A_k, B_k, s_k):
    """Eq. "grad_lora" for one task: returns (dA_k [h,r], dB_k [r,d])."""
    x_k, dh_k, A_k, B_k = _f64(x_k), _f64(dh_k), _f64(A_k), _f64(B_k)
    s_k = float(s_k)
    dA = s_k * (x_k.T @ (dh_k @ B_k.T))     # x_k^T dh_k B_k^T
    dB = s_k * (A_k.T @ (x_k.T @ dh_k))     # A_k^T x_k^T dh_k
    return dA, dB


def backward(X, W, dH, seg_offsets, A, B, s):
    """Eqs. "grad_lora" and "grad_output".

    Returns (dX [T,h], dA list, dB list).  The LoRA part of dX is added into
    the rows of dH W^T at the forward's split positions (the paper's "graph
    pruning": no zero-padded full-size intermediate).
    """
    X, W, dH = _f64(X), _f64(W), _f64(dH)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    T, h, d, K = _check(X, W, seg_offsets, A, B, s)
    assert dH.shape == (T, d)
    dA, dB = [], []
    # part one: adapter gradients, chunk by chunk
    for k in range(K):
        lo, hi = int(seg_offsets[k]), int(seg_offsets[k + 1])
        ga, gb = adapter_gradients(X[lo:hi], dH[lo:hi], A[k], B[k], s[k])
        dA.append(ga)
        dB.append(gb)
    # part two: dY = dH W^T once, then per-chunk dx_k added in place
    dX = dH @ W.T
    for k in range(K):
        lo, hi = int(seg_offsets[k]), int(seg_offsets[k + 1])
        dx_k = float(s[k]) * ((dH[lo:hi] @ B[k].T) @ A[k].T)
        dX[lo:hi] += dx_k
    return dX, dA, dB


def group_forward(X, Ws, seg_offsets, As, Bs, ss):
    """Several LoRA-wrapped projections applied to the same input (q, k, v of one
    attention block, gate and up of an MLP: section 4.1 puts adapters on q, k, v
    and o of every layer).  Projection p has its own W_p [h, d_p] and its own
    adapters A_{p,k}, B_{p,k}, s_{p,k}; all share X and the split positions.
    Each output is Eq. "forward" on its own: returns [(H_p, Z_p) for p].
    """
    assert len(Ws) == len(As) == len(Bs) == len(ss)
    return [forward(X, Ws[p], seg_offsets, As[p], Bs[p], ss[p]) for p in range(len(Ws))]


def group_backward(X, Ws, dHs, seg_offsets, As, Bs, ss):
    """Backward of `group_forward`.  X feeds every projection, so by the chain
    rule its gradient is the sum over the projections of Eq. "grad_output";
    the adapter gradients are Eq. "grad_lora" per projection.

    Returns (dX [T,h], dA[p][k], dB[p][k]).
    """
    assert len(Ws) == len(dHs) == len(As) == len(Bs) == len(ss)
    X = _f64(X)
    dX = np.zeros_like(X)
    dA, dB = [], []
    for p in range(len(Ws)):
        dx_p, da_p, db_p = backward(X, Ws[p], dHs[p], seg_offsets, As[p], Bs[p], ss[p])
        dX += dx_p
        dA.append(da_p)
        dB.append(db_p)
    return dX, dA, dB


def gather_rows_problem(rows, seg_offsets, T):
    """Host bookkeeping for row-sampled checks at sizes the full products are
    too slow for.  Every row of H and of dX depends on its own row of X / dH
    only, so the rows `rows` (sorted, unique) of the full problem equal the
    output of the smaller problem made of just those rows, with the segment
    offsets recomputed.  Returns (rows_sorted, new_offsets): the gathered
    matrix takes the rows in sorted order, which already is [uncovered rows
    before the first task | rows of task 0 | ... | uncovered rows after the
    last task], and new_offsets[k] is the position of the first gathered row
    that is >= seg_offsets[k].
    """
    rows = np.unique(np.asarray(rows, dtype=np.int64))
    assert rows.size == 0 or (rows[0] >= 0 and rows[-1] < T)
    new_off = [int(np.searchsorted(rows, int(o), side="left")) for o in seg_offsets]
    return rows, new_off


def flops(T, h, d, seg_offsets, ranks):
    """Useful floating-point operations of one forward + backward:
    4 T h d for the two base products plus 6 t_k r_k (h + d) per adapter."""
    f = 4.0 * T * h * d
    for k, r in enumerate(ranks):
        t = int(seg_offsets[k + 1]) - int(seg_offsets[k])
        f += 6.0 * t * r * (h + d)
    return f
