"""Pins for the CPU fp64 oracle: every check compares it with something that is
not the oracle's own code path -- hand-derived numbers, an element-wise scalar
evaluation written from the equations, closed forms, invariants the paper
states, and finite differences."""
import json
import os

import numpy as np
import pytest

from oracle import batchlora_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(rng, T, h, d, tokens, ranks, lead=0):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    assert off[-1] <= T
    X = rng.standard_normal((T, h))
    W = rng.standard_normal((h, d)) / np.sqrt(h)
    dH = rng.standard_normal((T, d))
    A = [rng.uniform(-1, 1, (h, r)) / np.sqrt(h) for r in ranks]
    B = [rng.standard_normal((r, d)) * 0.3 for r in ranks]
    s = [float(v) for v in rng.uniform(0.5, 3.0, len(ranks))]
    return X, W, dH, off, A, B, s


def _relerr(a, b):
    n = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (n if n > 0 else 1.0)


# ---------------------------------------------------------------- worked examples
@pytest.mark.parametrize("name", ["worked_example.json", "worked_example_rank2.json"])
def test_hand_derived_example(name):
    """Integers derived by hand from Eqs. forward / grad_lora / grad_output
    (section 3.3.1); the paper prints no worked example of its own."""
    with open(os.path.join(GOLDEN, name)) as f:
        g = json.load(f)
    A = [np.array(a, float) for a in g["A"]]
    B = [np.array(b, float) for b in g["B"]]
    H, Z = orc.forward(g["X"], g["W"], g["seg_offsets"], A, B, g["s"])
    dX, dA, dB = orc.backward(g["X"], g["W"], g["dH"], g["seg_offsets"], A, B, g["s"])
    assert np.array_equal(H, np.array(g["H"], float))
    assert np.array_equal(dX, np.array(g["dX"], float))
    for k in range(g["K"]):
        assert np.array_equal(Z[k], np.array(g["Z"][k], float))
        assert np.array_equal(dA[k], np.array(g["dA"][k], float))
        assert np.array_equal(dB[k], np.array(g["dB"][k], float))


# ---------------------------------------------------------------- scalar brute force
def _adapter_of_row(i, off):
    for k in range(len(off) - 1):
        if off[k] <= i < off[k + 1]:
            return k
    return -1


def test_scalar_brute_force():
    """Every output element from its own scalar sum, written from the
    equations element-wise (no matrix products, no shared helpers)."""
    rng = np.random.default_rng(5)
    T, h, d = 7, 3, 4
    X, W, dH, off, A, B, s = _rand_problem(rng, T, h, d, [2, 0, 3], [2, 1, 3], lead=1)
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    for i in range(T):
        k = _adapter_of_row(i, off)
        for j in range(d):
            v = sum(X[i, p] * W[p, j] for p in range(h))
            if k >= 0:
                r = A[k].shape[1]
                v += s[k] * sum(X[i, p] * A[k][p, q] * B[k][q, j] for p in range(h) for q in range(r))
            assert abs(v - H[i, j]) < 1e-12
        for p in range(h):
            v = sum(dH[i, j] * W[p, j] for j in range(d))
            if k >= 0:
                r = A[k].shape[1]
                v += s[k] * sum(dH[i, j] * B[k][q, j] * A[k][p, q] for j in range(d) for q in range(r))
            assert abs(v - dX[i, p]) < 1e-12
    for k in range(3):
        r = A[k].shape[1]
        rows = range(off[k], off[k + 1])
        for p in range(h):
            for q in range(r):
                v = s[k] * sum(X[i, p] * dH[i, j] * B[k][q, j] for i in rows for j in range(d))
                assert abs(v - dA[k][p, q]) < 1e-12
        for q in range(r):
            for j in range(d):
                v = s[k] * sum(A[k][p, q] * X[i, p] * dH[i, j] for i in rows for p in range(h))
                assert abs(v - dB[k][q, j]) < 1e-12
    # the empty segment (k=1) has zero gradients
    assert not dA[1].any() and not dB[1].any()


# ---------------------------------------------------------------- closed forms / special cases
def test_merged_weight_closed_form():
    """Eq. 1: x (W + s A B) = x W + s x A B, per adapter."""
    rng = np.random.default_rng(1)
    X, W, dH, off, A, B, s = _rand_problem(rng, 40, 12, 9, [13, 20, 7], [2, 4, 3])
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, _, _ = orc.backward(X, W, dH, off, A, B, s)
    for k in range(3):
        Wm = W + s[k] * (A[k] @ B[k])
        lo, hi = off[k], off[k + 1]
        assert _relerr(H[lo:hi], X[lo:hi] @ Wm) < 1e-13
        assert _relerr(dX[lo:hi], dH[lo:hi] @ Wm.T) < 1e-13


def test_B_zero_is_plain_linear():
    """Standard LoRA initialisation (B = 0): output and dX are the base
    model's, dA vanishes, dB = s (xA)^T dh."""
    rng = np.random.default_rng(2)
    X, W, dH, off, A, B, s = _rand_problem(rng, 30, 8, 6, [10, 20], [3, 2])
    B = [np.zeros_like(b) for b in B]
    H, Z = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    assert np.array_equal(H, X @ W)
    assert np.array_equal(dX, dH @ W.T)
    for k in range(2):
        assert not dA[k].any()
        lo, hi = off[k], off[k + 1]
        assert _relerr(dB[k], s[k] * (Z[k].T @ dH[lo:hi])) < 1e-13
        assert np.linalg.norm(dB[k]) > 0


def test_no_adapters_is_plain_gemm():
    """K = 0 reduces to a textbook matrix product; compared with an
    independently ordered triple loop."""
    rng = np.random.default_rng(3)
    T, h, d = 5, 4, 3
    X = rng.standard_normal((T, h)); W = rng.standard_normal((h, d)); dH = rng.standard_normal((T, d))
    H, Z = orc.forward(X, W, [0], [], [], [])
    dX, dA, dB = orc.backward(X, W, dH, [0], [], [], [])
    ref = np.zeros((T, d)); refx = np.zeros((T, h))
    for j in range(d):
        for p in range(h):
            for i in range(T):
                ref[i, j] += X[i, p] * W[p, j]
                refx[i, p] += dH[i, j] * W[p, j]
    assert np.allclose(H, ref, rtol=0, atol=1e-13) and np.allclose(dX, refx, rtol=0, atol=1e-13)
    assert Z == [] and dA == [] and dB == []


# ---------------------------------------------------------------- invariants from the paper
def test_batched_equals_sequential():
    """Listing 2 (batched) gives what Listing 1 (one adapter at a time) gives."""
    rng = np.random.default_rng(4)
    X, W, dH, off, A, B, s = _rand_problem(rng, 50, 10, 14, [16, 5, 29], [4, 1, 6])
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    for k in range(3):
        lo, hi = off[k], off[k + 1]
        Hk, _ = orc.forward(X[lo:hi], W, [0, hi - lo], [A[k]], [B[k]], [s[k]])
        dXk, dAk, dBk = orc.backward(X[lo:hi], W, dH[lo:hi], [0, hi - lo], [A[k]], [B[k]], [s[k]])
        assert _relerr(H[lo:hi], Hk) < 1e-14 and _relerr(dX[lo:hi], dXk) < 1e-14
        assert _relerr(dA[k], dAk[0]) < 1e-14 and _relerr(dB[k], dBk[0]) < 1e-14


def test_isolation_between_tasks():
    """Changing task j's data or adapter changes nothing that belongs to k != j."""
    rng = np.random.default_rng(6)
    X, W, dH, off, A, B, s = _rand_problem(rng, 36, 6, 5, [12, 12, 12], [2, 3, 2])
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    j = 1
    X2, dH2 = X.copy(), dH.copy()
    X2[off[j]:off[j + 1]] += 1.0
    dH2[off[j]:off[j + 1]] *= -2.0
    A2 = list(A); B2 = list(B); s2 = list(s)
    A2[j] = A[j] * 3 + 1; B2[j] = B[j] - 2; s2[j] = 7.0
    H2, _ = orc.forward(X2, W, off, A2, B2, s2)
    dX2, dA2, dB2 = orc.backward(X2, W, dH2, off, A2, B2, s2)
    for k in (0, 2):
        lo, hi = off[k], off[k + 1]
        assert np.array_equal(H[lo:hi], H2[lo:hi]) and np.array_equal(dX[lo:hi], dX2[lo:hi])
        assert np.array_equal(dA[k], dA2[k]) and np.array_equal(dB[k], dB2[k])
    lo, hi = off[j], off[j + 1]
    assert not np.array_equal(H[lo:hi], H2[lo:hi])


def test_segment_permutation_and_linearity_in_s():
    rng = np.random.default_rng(7)
    X, W, dH, off, A, B, s = _rand_problem(rng, 30, 5, 7, [8, 12, 10], [2, 2, 3])
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    perm = [2, 0, 1]
    rows = np.concatenate([np.arange(off[k], off[k + 1]) for k in perm])
    offp = [0]
    for k in perm:
        offp.append(offp[-1] + off[k + 1] - off[k])
    Hp, _ = orc.forward(X[rows], W, offp, [A[k] for k in perm], [B[k] for k in perm], [s[k] for k in perm])
    dXp, dAp, dBp = orc.backward(X[rows], W, dH[rows], offp, [A[k] for k in perm], [B[k] for k in perm],
                                 [s[k] for k in perm])
    assert _relerr(Hp, H[rows]) < 1e-14 and _relerr(dXp, dX[rows]) < 1e-14
    for i, k in enumerate(perm):
        assert _relerr(dAp[i], dA[k]) < 1e-14 and _relerr(dBp[i], dB[k]) < 1e-14
    # LoRA term, dA, dB are linear in s_k
    s2 = [2.0 * v for v in s]
    H2, _ = orc.forward(X, W, off, A, B, s2)
    dX2, dA2, dB2 = orc.backward(X, W, dH, off, A, B, s2)
    base, basex = X @ W, dH @ W.T
    assert _relerr(H2 - base, 2 * (H - base)) < 1e-12 and _relerr(dX2 - basex, 2 * (dX - basex)) < 1e-12
    for k in range(3):
        assert _relerr(dA2[k], 2 * dA[k]) < 1e-14 and _relerr(dB2[k], 2 * dB[k]) < 1e-14


def test_grad_B_two_orders_agree():
    """Eq. grad_lora prints dB = A^T x^T dh; it equals (x A)^T dh."""
    rng = np.random.default_rng(8)
    X, W, dH, off, A, B, s = _rand_problem(rng, 20, 6, 4, [20], [3])
    _, Z = orc.forward(X, W, off, A, B, s)
    _, dB = orc.adapter_gradients(X, dH, A[0], B[0], s[0])
    assert _relerr(dB, s[0] * (Z[0].T @ dH)) < 1e-13


# ---------------------------------------------------------------- finite differences
def test_finite_differences():
    """With L = sum(dH * H) (so dL/dH = dH exactly), central differences on
    every entry of X, A_k, B_k reproduce dX, dA_k, dB_k."""
    rng = np.random.default_rng(9)
    T, h, d = 9, 4, 5
    X, W, dH, off, A, B, s = _rand_problem(rng, T, h, d, [4, 3], [2, 3], lead=1)

    def loss(X_, A_, B_):
        H, _ = orc.forward(X_, W, off, A_, B_, s)
        return float((dH * H).sum())

    dX, dA, dB = orc.backward(X, W, dH, off, A, B, s)
    eps = 1e-6

    def fd(arr, setter):
        g = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = setter()
            arr[idx] = old - eps
            lm = setter()
            arr[idx] = old
            g[idx] = (lp - lm) / (2 * eps)
        return g

    gX = fd(X, lambda: loss(X, A, B))
    assert _relerr(gX, dX) < 1e-7
    for k in range(2):
        gA = fd(A[k], lambda: loss(X, A, B))
        gB = fd(B[k], lambda: loss(X, A, B))
        assert _relerr(gA, dA[k]) < 1e-7
        assert _relerr(gB, dB[k]) < 1e-7


# ---------------------------------------------------------------- row sampling bookkeeping
def test_row_sampled_problem_matches_full():
    """Rows of H and dX depend on their own input row only, so the gathered
    sub-problem reproduces the full problem's rows exactly."""
    rng = np.random.default_rng(10)
    T = 40
    X, W, dH, off, A, B, s = _rand_problem(rng, T, 6, 7, [10, 0, 15, 9], [2, 2, 1, 3], lead=3)
    H, _ = orc.forward(X, W, off, A, B, s)
    dX, _, _ = orc.backward(X, W, dH, off, A, B, s)
    rows = [0, 2, 3, 4, 12, 13, 20, 27, 28, 36, 37, 39]
    rs, off2 = orc.gather_rows_problem(rows, off, T)
    Hs, _ = orc.forward(X[rs], W, off2, A, B, s)
    dXs, _, _ = orc.backward(X[rs], W, dH[rs], off2, A, B, s)
    assert np.allclose(Hs, H[rs], rtol=0, atol=1e-13) and np.allclose(dXs, dX[rs], rtol=0, atol=1e-13)


def test_flops_formula():
    assert orc.flops(128, 256, 256, [0, 64, 128], [8, 8]) == 4 * 128 * 256 * 256 + 6 * 128 * 8 * 512


# ---------------------------------------------------------------- projection groups
def _rand_group(rng, T, h, ds, tokens, ranks_per_p, lead=0):
    off = [lead]
    for t in tokens:
        off.append(off[-1] + t)
    X = rng.standard_normal((T, h))
    Ws = [rng.standard_normal((h, d)) / np.sqrt(h) for d in ds]
    dHs = [rng.standard_normal((T, d)) for d in ds]
    As = [[rng.uniform(-1, 1, (h, r)) / np.sqrt(h) for r in ranks] for ranks in ranks_per_p]
    Bs = [[rng.standard_normal((r, d)) * 0.3 for r in ranks] for ranks, d in zip(ranks_per_p, ds)]
    ss = [[float(v) for v in rng.uniform(0.5, 3.0, len(ranks))] for ranks in ranks_per_p]
    return X, Ws, dHs, off, As, Bs, ss


def test_group_equals_concatenated_projection():
    """Projections that share X are one projection with the weights side by side:
    W = [W_0 | W_1 | ...], A_k = [A_0k | A_1k | ...], B_k block-diagonal (the scalings
    folded into its blocks).  Outputs are the column blocks, dX is the same matrix."""
    rng = np.random.default_rng(41)
    ds, rk = [5, 3, 4], [[2, 1, 3], [1, 1, 2], [3, 2, 1]]
    X, Ws, dHs, off, As, Bs, ss = _rand_group(rng, 17, 6, ds, [4, 0, 9], rk, lead=2)
    outs = orc.group_forward(X, Ws, off, As, Bs, ss)
    dX, dA, dB = orc.group_backward(X, Ws, dHs, off, As, Bs, ss)
    K, P = 3, 3
    Wc = np.concatenate(Ws, axis=1)
    dHc = np.concatenate(dHs, axis=1)
    Ac = [np.concatenate([As[p][k] for p in range(P)], axis=1) for k in range(K)]
    Bc = []
    for k in range(K):
        rows = []
        for p in range(P):
            blocks = [ss[p][k] * Bs[p][k] if q == p else np.zeros((rk[p][k], ds[q])) for q in range(P)]
            rows.append(np.concatenate(blocks, axis=1))
        Bc.append(np.concatenate(rows, axis=0))
    Hc, _ = orc.forward(X, Wc, off, Ac, Bc, [1.0] * K)
    dXc, dAc, dBc = orc.backward(X, Wc, dHc, off, Ac, Bc, [1.0] * K)
    c0 = np.cumsum([0] + ds)
    for p in range(P):
        assert _relerr(outs[p][0], Hc[:, c0[p]:c0[p + 1]]) < 1e-13
    assert _relerr(dX, dXc) < 1e-13
    for k in range(K):
        r0 = np.cumsum([0] + [rk[p][k] for p in range(P)])
        for p in range(P):
            # dA of the concatenation holds the projections' dA side by side
            assert _relerr(dA[p][k], dAc[k][:, r0[p]:r0[p + 1]]) < 1e-12
            # its dB holds (x A_pk)^T dH_p on the diagonal blocks, i.e. dB_pk without the scaling
            assert _relerr(dB[p][k], ss[p][k] * dBc[k][r0[p]:r0[p + 1], c0[p]:c0[p + 1]]) < 1e-12


def test_group_scalar_brute_force():
    """dX[i,c] = sum_p sum_j dH_p[i,j] (W_p[c,j] + s_pk sum_q A_pk[c,q] B_pk[q,j]), element by element."""
    rng = np.random.default_rng(43)
    ds, rk = [3, 2], [[2, 1], [1, 2]]
    X, Ws, dHs, off, As, Bs, ss = _rand_group(rng, 7, 4, ds, [3, 3], rk, lead=1)
    dX, _, _ = orc.group_backward(X, Ws, dHs, off, As, Bs, ss)
    for i in range(7):
        k = _adapter_of_row(i, off)
        for c in range(4):
            acc = 0.0
            for p in range(2):
                for j in range(ds[p]):
                    w = Ws[p][c, j]
                    if k >= 0:
                        for q in range(rk[p][k]):
                            w += ss[p][k] * As[p][k][c, q] * Bs[p][k][q, j]
                    acc += dHs[p][i, j] * w
            assert abs(dX[i, c] - acc) < 1e-12


def test_group_of_worked_example_copies():
    """Two copies of the hand-derived example sharing X, the second one's output gradient
    scaled by -3: outputs repeat, adapter gradients scale, dX = (1 - 3) dX by linearity."""
    with open(os.path.join(GOLDEN, "worked_example.json")) as f:
        g = json.load(f)
    A = [np.array(a, float) for a in g["A"]]
    B = [np.array(b, float) for b in g["B"]]
    dH = np.array(g["dH"], float)
    outs = orc.group_forward(g["X"], [g["W"]] * 2, g["seg_offsets"], [A, A], [B, B], [g["s"], g["s"]])
    dX, dA, dB = orc.group_backward(g["X"], [g["W"]] * 2, [dH, -3.0 * dH], g["seg_offsets"], [A, A], [B, B],
                                    [g["s"], g["s"]])
    for p in range(2):
        assert np.array_equal(outs[p][0], np.array(g["H"], float))
    assert np.array_equal(dX, -2.0 * np.array(g["dX"], float))
    for k in range(g["K"]):
        assert np.array_equal(dA[0][k], np.array(g["dA"][k], float))
        assert np.array_equal(dA[1][k], -3.0 * np.array(g["dA"][k], float))
        assert np.array_equal(dB[1][k], -3.0 * np.array(g["dB"][k], float))


def test_group_finite_differences():
    """Central differences of L = sum_p sum(dH_p * H_p) in X and in one adapter of each projection."""
    rng = np.random.default_rng(47)
    ds, rk = [4, 3], [[2, 3], [1, 2]]
    X, Ws, dHs, off, As, Bs, ss = _rand_group(rng, 9, 5, ds, [4, 5], rk)
    dX, dA, dB = orc.group_backward(X, Ws, dHs, off, As, Bs, ss)

    def loss(Xv, Av, Bv):
        outs = orc.group_forward(Xv, Ws, off, Av, Bv, ss)
        return sum(float(np.sum(dHs[p] * outs[p][0])) for p in range(2))

    eps = 1e-6
    num = np.zeros_like(X)
    for i in range(X.shape[0]):
        for c in range(X.shape[1]):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, c] += eps
            Xm[i, c] -= eps
            num[i, c] = (loss(Xp, As, Bs) - loss(Xm, As, Bs)) / (2 * eps)
    assert _relerr(num, dX) < 1e-7
    for p, k in ((0, 1), (1, 0)):
        numA = np.zeros_like(As[p][k])
        for i in range(numA.shape[0]):
            for q in range(numA.shape[1]):
                Ap = [[a.copy() for a in row] for row in As]
                Am = [[a.copy() for a in row] for row in As]
                Ap[p][k][i, q] += eps
                Am[p][k][i, q] -= eps
                numA[i, q] = (loss(X, Ap, Bs) - loss(X, Am, Bs)) / (2 * eps)
        assert _relerr(numA, dA[p][k]) < 1e-7
        numB = np.zeros_like(Bs[p][k])
        for q in range(numB.shape[0]):
            for j in range(numB.shape[1]):
                Bp = [[b.copy() for b in row] for row in Bs]
                Bm = [[b.copy() for b in row] for row in Bs]
                Bp[p][k][q, j] += eps
                Bm[p][k][q, j] -= eps
                numB[q, j] = (loss(X, As, Bp) - loss(X, As, Bm)) / (2 * eps)
        assert _relerr(numB, dB[p][k]) < 1e-7
