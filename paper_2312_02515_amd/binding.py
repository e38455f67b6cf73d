"""Thin ctypes binding over the C ABI of libmlora.so (see include/mlora.h, include/mlora_testing.h).

Argument marshalling only: every arithmetic step runs in the library's HIP
kernels.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmlora.so")

MLORA_BF16 = 0
MLORA_F32 = 1
MLORA_MAX_ADAPTERS = 64
MLORA_MAX_RANK = 128
MLORA_MAX_GROUP = 4

STATUS_NAMES = {0: "MLORA_OK", 1: "MLORA_ERR_NULL", 2: "MLORA_ERR_SHAPE", 3: "MLORA_ERR_SEGMENTS",
                4: "MLORA_ERR_RANK", 5: "MLORA_ERR_DTYPE", 6: "MLORA_ERR_WORKSPACE", 7: "MLORA_ERR_HIP"}

EXPORTS = ["mlora_lora_saved_bytes", "mlora_lora_workspace_bytes", "mlora_lora_validate", "mlora_lora_fwd",
           "mlora_lora_bwd", "mlora_lora_recompute_workspace_bytes", "mlora_lora_fwd_nosave",
           "mlora_lora_bwd_recompute", "mlora_lora_group_validate", "mlora_lora_group_workspace_bytes",
           "mlora_lora_group_fwd", "mlora_lora_group_bwd", "mlora_status_string", "mlora_last_hip_error",
           "mlora_lora_kernel_path", "mlora_lora_bwd_static", "mlora_w8_quantize", "mlora_w8_dequantize",
           "mlora_lora_w8_workspace_bytes", "mlora_lora_fwd_w8", "mlora_lora_bwd_w8"]
MLORA_STATIC_SCRATCH_BYTES = 32 << 20
# include/mlora_testing.h: test and measurement switches
TESTING_EXPORTS = ["mlora_set_kernel_path", "mlora_profile_kernels", "mlora_profile_kernels_read"]


class MloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.mlora_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg}); hip error {lib.mlora_last_hip_error()}")


class mlora_problem(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("h", ctypes.c_int64), ("d", ctypes.c_int64),
                ("K", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("seg_offsets", ctypes.POINTER(ctypes.c_int64)),
                ("ranks", ctypes.POINTER(ctypes.c_int32)),
                ("scalings", ctypes.POINTER(ctypes.c_float)),
                ("A", ctypes.POINTER(ctypes.c_void_p)),
                ("B", ctypes.POINTER(ctypes.c_void_p)),
                ("W", ctypes.c_void_p)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path.")
    l = ctypes.CDLL(LIB_PATH)
    pp = ctypes.POINTER(mlora_problem)
    l.mlora_lora_saved_bytes.restype = ctypes.c_size_t
    l.mlora_lora_saved_bytes.argtypes = [pp]
    l.mlora_lora_workspace_bytes.restype = ctypes.c_size_t
    l.mlora_lora_workspace_bytes.argtypes = [pp]
    l.mlora_lora_validate.restype = ctypes.c_int
    l.mlora_lora_validate.argtypes = [pp]
    l.mlora_lora_fwd.restype = ctypes.c_int
    l.mlora_lora_fwd.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_size_t, ctypes.c_void_p]
    l.mlora_lora_bwd.restype = ctypes.c_int
    l.mlora_lora_bwd.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    l.mlora_lora_bwd_static.restype = ctypes.c_int
    l.mlora_lora_bwd_static.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                        ctypes.c_void_p]
    l.mlora_lora_recompute_workspace_bytes.restype = ctypes.c_size_t
    l.mlora_lora_recompute_workspace_bytes.argtypes = [pp]
    l.mlora_w8_quantize.restype = ctypes.c_int
    l.mlora_w8_quantize.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p]
    l.mlora_w8_dequantize.restype = ctypes.c_int
    l.mlora_w8_dequantize.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_void_p]
    l.mlora_lora_w8_workspace_bytes.restype = ctypes.c_size_t
    l.mlora_lora_w8_workspace_bytes.argtypes = [pp]
    l.mlora_lora_fwd_w8.restype = ctypes.c_int
    l.mlora_lora_fwd_w8.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    l.mlora_lora_bwd_w8.restype = ctypes.c_int
    l.mlora_lora_bwd_w8.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p),
                                    ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                    ctypes.c_void_p]
    l.mlora_lora_fwd_nosave.restype = ctypes.c_int
    l.mlora_lora_fwd_nosave.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.c_void_p]
    l.mlora_lora_bwd_recompute.restype = ctypes.c_int
    l.mlora_lora_bwd_recompute.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                                           ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    ppp = ctypes.POINTER(pp)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    l.mlora_lora_group_validate.restype = ctypes.c_int
    l.mlora_lora_group_validate.argtypes = [ppp, ctypes.c_int]
    l.mlora_lora_group_workspace_bytes.restype = ctypes.c_size_t
    l.mlora_lora_group_workspace_bytes.argtypes = [ppp, ctypes.c_int]
    l.mlora_lora_group_fwd.restype = ctypes.c_int
    l.mlora_lora_group_fwd.argtypes = [ppp, ctypes.c_int, ctypes.c_void_p, vpp, vpp, ctypes.c_void_p, ctypes.c_size_t,
                                       ctypes.c_void_p]
    l.mlora_lora_group_bwd.restype = ctypes.c_int
    l.mlora_lora_group_bwd.argtypes = [ppp, ctypes.c_int, ctypes.c_void_p, vpp, vpp, ctypes.c_void_p,
                                       ctypes.POINTER(vpp), ctypes.POINTER(vpp), ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_size_t, ctypes.c_void_p]
    l.mlora_status_string.restype = ctypes.c_char_p
    l.mlora_status_string.argtypes = [ctypes.c_int]
    l.mlora_last_hip_error.restype = ctypes.c_int
    l.mlora_last_hip_error.argtypes = []
    l.mlora_lora_kernel_path.restype = ctypes.c_int
    l.mlora_lora_kernel_path.argtypes = [pp]
    l.mlora_set_kernel_path.restype = ctypes.c_int
    l.mlora_set_kernel_path.argtypes = [ctypes.c_int]
    l.mlora_profile_kernels.restype = ctypes.c_int
    l.mlora_profile_kernels.argtypes = [ctypes.c_int]
    l.mlora_profile_kernels_read.restype = ctypes.c_int
    l.mlora_profile_kernels_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_int)]
    return l


lib = _load()


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return MLORA_BF16
    if dt == torch.float32:
        return MLORA_F32
    raise TypeError(f"unsupported dtype {dt}")


class Problem:
    """Host-side description of one call: owns the ctypes arrays the struct points to
    and keeps the adapter tensors alive.  W may be None for the calls that take the weight in
    its 8-bit code (then `dtype` and `device` say what W would have been)."""

    def __init__(self, T: int, h: int, d: int, W: Optional[torch.Tensor], seg_offsets: Sequence[int],
                 ranks: Sequence[int], scalings: Sequence[float], A: Sequence[torch.Tensor], B: Sequence[torch.Tensor],
                 dtype: Optional[torch.dtype] = None, device=None):
        K = len(ranks)
        self.T, self.h, self.d, self.K = int(T), int(h), int(d), K
        self.ranks = [int(r) for r in ranks]
        self.W, self.A, self.B = W, list(A), list(B)
        self.torch_dtype = W.dtype if W is not None else dtype
        self.device = W.device if W is not None else torch.device(device)
        self._off = (ctypes.c_int64 * (K + 1))(*[int(o) for o in seg_offsets])
        self._ranks = (ctypes.c_int32 * max(K, 1))(*self.ranks)
        self._s = (ctypes.c_float * max(K, 1))(*[float(s) for s in scalings])
        self._A = (ctypes.c_void_p * max(K, 1))(*[a.data_ptr() for a in A])
        self._B = (ctypes.c_void_p * max(K, 1))(*[b.data_ptr() for b in B])
        self.c = mlora_problem(T=self.T, h=self.h, d=self.d, K=K, dtype=_dtype_code(self.torch_dtype),
                               seg_offsets=ctypes.cast(self._off, ctypes.POINTER(ctypes.c_int64)),
                               ranks=ctypes.cast(self._ranks, ctypes.POINTER(ctypes.c_int32)),
                               scalings=ctypes.cast(self._s, ctypes.POINTER(ctypes.c_float)),
                               A=ctypes.cast(self._A, ctypes.POINTER(ctypes.c_void_p)),
                               B=ctypes.cast(self._B, ctypes.POINTER(ctypes.c_void_p)),
                               W=W.data_ptr() if W is not None else None)

    def saved_bytes(self) -> int:
        return int(lib.mlora_lora_saved_bytes(ctypes.byref(self.c)))

    def workspace_bytes(self) -> int:
        return int(lib.mlora_lora_workspace_bytes(ctypes.byref(self.c)))

    def recompute_workspace_bytes(self) -> int:
        return int(lib.mlora_lora_recompute_workspace_bytes(ctypes.byref(self.c)))

    def alloc_recompute_workspace(self) -> torch.Tensor:
        return torch.empty(self.recompute_workspace_bytes(), dtype=torch.uint8, device=self.device)

    def validate(self) -> int:
        return int(lib.mlora_lora_validate(ctypes.byref(self.c)))

    def kernel_path(self) -> int:
        """0 = MFMA kernels; bit 0 / bit 1 = generic kernels for the base / low-rank products."""
        return int(lib.mlora_lora_kernel_path(ctypes.byref(self.c)))

    def alloc_saved(self) -> torch.Tensor:
        return torch.empty(self.saved_bytes(), dtype=torch.uint8, device=self.device)

    def alloc_workspace(self) -> torch.Tensor:
        return torch.empty(self.workspace_bytes(), dtype=torch.uint8, device=self.device)

    def w8_workspace_bytes(self) -> int:
        return int(lib.mlora_lora_w8_workspace_bytes(ctypes.byref(self.c)))

    def alloc_w8_workspace(self) -> torch.Tensor:
        return torch.empty(self.w8_workspace_bytes(), dtype=torch.uint8, device=self.device)

    def alloc_grads(self):
        dA = [torch.empty((self.h, r), dtype=torch.float32, device=self.device) for r in self.ranks]
        dB = [torch.empty((r, self.d), dtype=torch.float32, device=self.device) for r in self.ranks]
        return dA, dB


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def mlora_lora_fwd(prob: Problem, X: torch.Tensor, Y: torch.Tensor, saved: torch.Tensor, workspace: torch.Tensor,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    """Y = X W + rows_k(s_k x_k A_k B_k); fills `saved` for the backward call."""
    st = lib.mlora_lora_fwd(ctypes.byref(prob.c), X.data_ptr(), Y.data_ptr(), saved.data_ptr(), workspace.data_ptr(),
                            workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_fwd")


def mlora_lora_bwd(prob: Problem, X: torch.Tensor, dY: torch.Tensor, saved: torch.Tensor,
                   dX: Optional[torch.Tensor], dA: List[torch.Tensor], dB: List[torch.Tensor], accumulate: bool,
                   workspace: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """dX = dY W^T + rows_k(s_k dy_k B_k^T A_k^T); dA_k, dB_k as in Eq. grad_lora."""
    K = prob.K
    pa = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dA])
    pb = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dB])
    st = lib.mlora_lora_bwd(ctypes.byref(prob.c), X.data_ptr(), dY.data_ptr(), saved.data_ptr(),
                            dX.data_ptr() if dX is not None else None,
                            ctypes.cast(pa, ctypes.POINTER(ctypes.c_void_p)),
                            ctypes.cast(pb, ctypes.POINTER(ctypes.c_void_p)), 1 if accumulate else 0,
                            workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                            _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_bwd")


def mlora_lora_bwd_static(prob: Problem, X: torch.Tensor, dY: torch.Tensor, saved: torch.Tensor,
                          dX: Optional[torch.Tensor], dA: List[torch.Tensor], dB: List[torch.Tensor], accumulate: bool,
                          stream: Optional[torch.cuda.Stream] = None) -> None:
    """mlora_lora_bwd with the library's own fixed scratch array instead of a workspace."""
    K = prob.K
    pa = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dA])
    pb = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dB])
    st = lib.mlora_lora_bwd_static(ctypes.byref(prob.c), X.data_ptr(), dY.data_ptr(), saved.data_ptr(),
                                   dX.data_ptr() if dX is not None else None,
                                   ctypes.cast(pa, ctypes.POINTER(ctypes.c_void_p)),
                                   ctypes.cast(pb, ctypes.POINTER(ctypes.c_void_p)), 1 if accumulate else 0,
                                   _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_bwd_static")


def mlora_w8_quantize(W: torch.Tensor, stream: Optional[torch.cuda.Stream] = None):
    """Column-wise absmax code of W [h, d]: returns (Wq int8 [h, d], c float32 [d])."""
    h, d = W.shape
    Wq = torch.empty((h, d), dtype=torch.int8, device=W.device)
    c = torch.empty((d,), dtype=torch.float32, device=W.device)
    st = lib.mlora_w8_quantize(W.data_ptr(), _dtype_code(W.dtype), h, d, Wq.data_ptr(), c.data_ptr(),
                               _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_w8_quantize")
    return Wq, c


def mlora_w8_dequantize(Wq: torch.Tensor, c: torch.Tensor, dtype: torch.dtype,
                        stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """W^ = Wq c_j in the storage type `dtype`."""
    h, d = Wq.shape
    out = torch.empty((h, d), dtype=dtype, device=Wq.device)
    st = lib.mlora_w8_dequantize(Wq.data_ptr(), c.data_ptr(), _dtype_code(dtype), h, d, out.data_ptr(),
                                 _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_w8_dequantize")
    return out


def mlora_lora_fwd_w8(prob: Problem, Wq: torch.Tensor, c: torch.Tensor, X: torch.Tensor, Y: torch.Tensor,
                      saved: torch.Tensor, workspace: torch.Tensor,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
    """mlora_lora_fwd with the frozen weight given as its 8-bit code (Wq, c)."""
    st = lib.mlora_lora_fwd_w8(ctypes.byref(prob.c), Wq.data_ptr(), c.data_ptr(), X.data_ptr(), Y.data_ptr(),
                               saved.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                               _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_fwd_w8")


def mlora_lora_bwd_w8(prob: Problem, Wq: torch.Tensor, c: torch.Tensor, X: torch.Tensor, dY: torch.Tensor,
                      saved: torch.Tensor, dX: Optional[torch.Tensor], dA: List[torch.Tensor], dB: List[torch.Tensor],
                      accumulate: bool, workspace: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """mlora_lora_bwd with the frozen weight given as its 8-bit code (Wq, c)."""
    K = prob.K
    pa = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dA])
    pb = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dB])
    st = lib.mlora_lora_bwd_w8(ctypes.byref(prob.c), Wq.data_ptr(), c.data_ptr(), X.data_ptr(), dY.data_ptr(),
                               saved.data_ptr(), dX.data_ptr() if dX is not None else None,
                               ctypes.cast(pa, ctypes.POINTER(ctypes.c_void_p)),
                               ctypes.cast(pb, ctypes.POINTER(ctypes.c_void_p)), 1 if accumulate else 0,
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                               _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_bwd_w8")


def mlora_lora_fwd_nosave(prob: Problem, X: torch.Tensor, Y: torch.Tensor, workspace: torch.Tensor,
                          stream: Optional[torch.cuda.Stream] = None) -> None:
    """Forward of the activation-recompute variant: as mlora_lora_fwd, nothing saved."""
    st = lib.mlora_lora_fwd_nosave(ctypes.byref(prob.c), X.data_ptr(), Y.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_fwd_nosave")


def mlora_lora_bwd_recompute(prob: Problem, X: torch.Tensor, dY: torch.Tensor, dX: Optional[torch.Tensor],
                             dA: List[torch.Tensor], dB: List[torch.Tensor], accumulate: bool,
                             workspace: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Backward of the activation-recompute variant: recomputes s_k x_k A_k from X."""
    K = prob.K
    pa = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dA])
    pb = (ctypes.c_void_p * max(K, 1))(*[t.data_ptr() for t in dB])
    st = lib.mlora_lora_bwd_recompute(ctypes.byref(prob.c), X.data_ptr(), dY.data_ptr(),
                                      dX.data_ptr() if dX is not None else None,
                                      ctypes.cast(pa, ctypes.POINTER(ctypes.c_void_p)),
                                      ctypes.cast(pb, ctypes.POINTER(ctypes.c_void_p)), 1 if accumulate else 0,
                                      workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                      _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_bwd_recompute")


class Group:
    """Projections that share their input: a host array of pointers to their problems."""

    def __init__(self, problems: Sequence[Problem]):
        self.problems = list(problems)
        self.P = len(self.problems)
        self._arr = (ctypes.POINTER(mlora_problem) * max(self.P, 1))(*[ctypes.pointer(p.c) for p in self.problems])
        self.c = ctypes.cast(self._arr, ctypes.POINTER(ctypes.POINTER(mlora_problem)))

    def validate(self) -> int:
        return int(lib.mlora_lora_group_validate(self.c, self.P))

    def workspace_bytes(self) -> int:
        return int(lib.mlora_lora_group_workspace_bytes(self.c, self.P))

    def alloc_workspace(self) -> torch.Tensor:
        return torch.empty(self.workspace_bytes(), dtype=torch.uint8, device=self.problems[0].device)


def _ptr_array(tensors):
    arr = (ctypes.c_void_p * max(len(tensors), 1))(*[t.data_ptr() for t in tensors])
    return arr, ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))


def mlora_lora_group_fwd(group: Group, X: torch.Tensor, Y: Sequence[torch.Tensor], saved: Sequence[torch.Tensor],
                         workspace: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Y[p] = X W_p + rows_k(s_pk x_k A_pk B_pk) for every projection p of the group."""
    ky, py = _ptr_array(Y)
    ks, ps_ = _ptr_array(saved)
    st = lib.mlora_lora_group_fwd(group.c, group.P, X.data_ptr(), py, ps_, workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_group_fwd")


def mlora_lora_group_bwd(group: Group, X: torch.Tensor, dY: Sequence[torch.Tensor], saved: Sequence[torch.Tensor],
                         dX: Optional[torch.Tensor], dA: Sequence[List[torch.Tensor]],
                         dB: Sequence[List[torch.Tensor]], accumulate: bool, workspace: torch.Tensor,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """One dX = sum_p (dY_p W_p^T + LoRA part); dA[p][k], dB[p][k] per projection."""
    kd, pd = _ptr_array(dY)
    ks, ps_ = _ptr_array(saved)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    keep, rows_a, rows_b = [], [], []
    for p in range(group.P):
        a, pa = _ptr_array(dA[p])
        b, pb = _ptr_array(dB[p])
        keep += [a, b]
        rows_a.append(pa)
        rows_b.append(pb)
    ta = (vpp * max(group.P, 1))(*rows_a)
    tb = (vpp * max(group.P, 1))(*rows_b)
    st = lib.mlora_lora_group_bwd(group.c, group.P, X.data_ptr(), pd, ps_, dX.data_ptr() if dX is not None else None,
                                  ctypes.cast(ta, ctypes.POINTER(vpp)), ctypes.cast(tb, ctypes.POINTER(vpp)),
                                  1 if accumulate else 0, workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise MloraError(st, "mlora_lora_group_bwd")


def set_kernel_path(path: int) -> int:
    return int(lib.mlora_set_kernel_path(int(path)))


PROFILE_KINDS = ("gemm", "rows", "grad")


def profile_kernels(enable: bool) -> bool:
    return bool(lib.mlora_profile_kernels(1 if enable else 0))


def profile_kernels_read():
    """{kind: (total ms, total algorithmic units, launches)} of the MFMA kernels since the last read;
    units are flops for "gemm" and bytes for "rows" (s x A, s dy B^T) and "grad" (dA, dB)."""
    n = len(PROFILE_KINDS)
    ms, un, cnt = (ctypes.c_double * n)(), (ctypes.c_double * n)(), (ctypes.c_int * n)()
    st = lib.mlora_profile_kernels_read(ms, un, cnt)
    if st != 0:
        raise MloraError(st, "mlora_profile_kernels_read")
    return {k: (ms[i], un[i], cnt[i]) for i, k in enumerate(PROFILE_KINDS)}
