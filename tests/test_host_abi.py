"""CPU-only checks of the C-ABI library: it loads, exports every function that
include/mlora.h declares, and turns every invalid argument into its error code
before any GPU work (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mb():
    from paper_2312_02515_amd import binding
    return binding


@pytest.mark.parametrize("header,exports", [("mlora.h", "EXPORTS"), ("mlora_testing.h", "TESTING_EXPORTS")])
def test_exports_match_header(mb, header, exports):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(mlora_[a-z0-9_]+)\s*\(", text))
    assert declared == set(getattr(mb, exports))
    for name in declared:
        assert hasattr(mb.lib, name), name


def test_every_header_is_covered(mb):
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["mlora.h", "mlora_testing.h"]


def test_header_is_plain_c_and_links(mb, tmp_path):
    """include/mlora.h compiles as C (gcc, -std=c99 -pedantic) and a C program linked against the
    library can call the argument-checking entry points."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "abi_check")
    libdir = os.path.dirname(mb.LIB_PATH)
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "abi_check.c"), "-o", exe, "-L", libdir, "-l:libmlora.so",
           "-Wl,-rpath," + libdir]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "abi_check: ok" in r.stdout, r.stdout + r.stderr


def test_status_strings(mb):
    for code in range(8):
        assert mb.lib.mlora_status_string(code)
    assert mb.lib.mlora_status_string(99) == b"unknown status"


class _FakeTensor:
    """Stands in for a device tensor: only its address is marshalled."""

    def __init__(self, addr=0x1000):
        self._a = addr
        import torch
        self.dtype = torch.bfloat16
        self.device = "cpu"

    def data_ptr(self):
        return self._a


def _problem(mb, T=64, h=32, d=48, off=(0, 32, 64), ranks=(8, 4), s=(2.0, 2.0), null_A=False):
    W = _FakeTensor()
    A = [_FakeTensor(0 if null_A else 0x2000) for _ in ranks]
    B = [_FakeTensor(0x3000) for _ in ranks]
    return mb.Problem(T, h, d, W, off, ranks, s, A, B)


def test_valid_problem_sizes(mb):
    p = _problem(mb)
    assert p.validate() == 0
    assert p.saved_bytes() >= 64 * 16 * 2
    assert p.workspace_bytes() >= 64 * 16 * 2


@pytest.mark.parametrize("kw,code", [
    (dict(off=(0, 40, 30)), 3),            # not monotone
    (dict(off=(0, 32, 65)), 3),            # beyond T
    (dict(off=(-1, 32, 64)), 3),
    (dict(ranks=(0, 4)), 4),
    (dict(ranks=(8, 129)), 4),
    (dict(h=0), 2),
    (dict(T=-1), 2),
    (dict(d=(1 << 22) + 64), 2),           # feature sizes beyond 4 Mi
    (dict(T=1 << 31, off=(0, 32, 64)), 2),  # too many rows
    (dict(T=(1 << 31) - 2048, d=1 << 22, off=(0, 32, 64)), 2),  # more than 2^31 tiles
    (dict(null_A=True), 1),
])
def test_validation_codes(mb, kw, code):
    p = _problem(mb, **kw)
    assert p.validate() == code
    assert p.saved_bytes() == 0 and p.workspace_bytes() == 0


def test_too_many_adapters_and_dtype(mb):
    K = 65
    p = _problem(mb, T=65, off=tuple(range(K + 1)), ranks=(4,) * K, s=(1.0,) * K)
    assert p.validate() == 2
    p = _problem(mb)
    p.c.dtype = 7
    assert p.validate() == 5
    p.c.dtype = 0
    p.c.W = None
    assert p.validate() == 1
    assert mb.lib.mlora_lora_validate(None) == 1


def test_entry_points_reject_before_launch(mb):
    """NULL buffers and a short workspace are reported without touching the GPU."""
    p = _problem(mb)
    ws = p.workspace_bytes()
    f = mb.lib.mlora_lora_fwd
    assert f(ctypes.byref(p.c), None, 0x10, 0x20, 0x30, ws, None) == 1
    assert f(ctypes.byref(p.c), 0x10, 0x20, 0x30, None, ws, None) == 6
    assert f(ctypes.byref(p.c), 0x10, 0x20, 0x30, 0x40, ws - 1, None) == 6
    b = mb.lib.mlora_lora_bwd
    arr = (ctypes.c_void_p * 2)(0x50, 0x60)
    pa = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert b(ctypes.byref(p.c), 0x10, None, 0x20, 0x30, pa, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x10, 0x11, 0x20, 0x30, None, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x10, 0x11, 0x20, 0x30, pa, pa, 0, 0x40, 0, None) == 6
    bad = _problem(mb, off=(0, 40, 30))
    assert f(ctypes.byref(bad.c), 0x10, 0x20, 0x30, 0x40, 1 << 20, None) == 3


def test_recompute_entry_points_reject_before_launch(mb):
    """The activation-recompute pair: twice the workspace, same argument checks."""
    p = _problem(mb)
    ws = p.recompute_workspace_bytes()
    assert ws == 2 * p.workspace_bytes()
    f = mb.lib.mlora_lora_fwd_nosave
    assert f(ctypes.byref(p.c), None, 0x20, 0x40, ws, None) == 1
    assert f(ctypes.byref(p.c), 0x10, 0x20, 0x40, p.workspace_bytes(), None) == 6
    assert f(ctypes.byref(p.c), 0x10, 0x20, None, ws, None) == 6
    b = mb.lib.mlora_lora_bwd_recompute
    arr = (ctypes.c_void_p * 2)(0x50, 0x60)
    pa = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert b(ctypes.byref(p.c), 0x10, None, 0x30, pa, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x10, 0x11, 0x30, pa, None, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x10, 0x11, 0x30, pa, pa, 0, 0x40, ws - 1, None) == 6
    bad = _problem(mb, off=(0, 40, 30))
    assert b(ctypes.byref(bad.c), 0x10, 0x11, 0x30, pa, pa, 0, 0x40, 1 << 20, None) == 3
    assert mb.lib.mlora_lora_recompute_workspace_bytes(ctypes.byref(bad.c)) == 0


def test_w8_entry_points_reject_before_launch(mb):
    """The 8-bit-weight calls: p->W is ignored, the workspace also holds the decoded weight, and
    NULL codes, NULL buffers and a short workspace are reported without touching the GPU."""
    p = _problem(mb)
    plain = p.workspace_bytes()
    ws = p.w8_workspace_bytes()
    assert ws == plain + (32 * 48 * 2 + 255) // 256 * 256
    p.c.W = None                      # not needed by the w8 calls ...
    assert p.w8_workspace_bytes() == ws
    assert p.validate() == 1          # ... while the plain calls insist on it
    f = mb.lib.mlora_lora_fwd_w8
    assert f(ctypes.byref(p.c), None, 0x70, 0x10, 0x20, 0x30, 0x40, ws, None) == 1
    assert f(ctypes.byref(p.c), 0x60, None, 0x10, 0x20, 0x30, 0x40, ws, None) == 1
    assert f(ctypes.byref(p.c), 0x60, 0x70, None, 0x20, 0x30, 0x40, ws, None) == 1
    assert f(ctypes.byref(p.c), 0x60, 0x70, 0x10, 0x20, 0x30, None, ws, None) == 6
    assert f(ctypes.byref(p.c), 0x60, 0x70, 0x10, 0x20, 0x30, 0x40, ws - 1, None) == 6
    assert f(ctypes.byref(p.c), 0x60, 0x70, 0x10, 0x20, 0x30, 0x40, plain, None) == 6
    assert f(None, 0x60, 0x70, 0x10, 0x20, 0x30, 0x40, ws, None) == 1
    b = mb.lib.mlora_lora_bwd_w8
    arr = (ctypes.c_void_p * 2)(0x50, 0x60)
    pa = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert b(ctypes.byref(p.c), None, 0x70, 0x10, 0x11, 0x20, 0x30, pa, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x60, 0x70, 0x10, None, 0x20, 0x30, pa, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x60, 0x70, 0x10, 0x11, 0x20, 0x30, None, pa, 0, 0x40, ws, None) == 1
    assert b(ctypes.byref(p.c), 0x60, 0x70, 0x10, 0x11, 0x20, 0x30, pa, pa, 0, 0x40, ws - 1, None) == 6
    bad = _problem(mb, off=(0, 40, 30))
    assert bad.w8_workspace_bytes() == 0
    assert f(ctypes.byref(bad.c), 0x60, 0x70, 0x10, 0x20, 0x30, 0x40, 1 << 20, None) == 3
    assert b(ctypes.byref(bad.c), 0x60, 0x70, 0x10, 0x11, 0x20, 0x30, pa, pa, 0, 0x40, 1 << 20, None) == 3
    empty = _problem(mb, T=0, off=(0, 0, 0))
    assert f(ctypes.byref(empty.c), 0x60, 0x70, None, None, None, None, 0, None) == 0
    q, dq = mb.lib.mlora_w8_quantize, mb.lib.mlora_w8_dequantize
    assert q(None, 0, 8, 8, 0x10, 0x20, None) == 1 and q(0x10, 0, 8, 8, None, 0x20, None) == 1
    assert q(0x10, 3, 8, 8, 0x20, 0x30, None) == 5
    assert q(0x10, 0, 0, 8, 0x20, 0x30, None) == 2 and q(0x10, 0, 8, (1 << 22) + 1, 0x20, 0x30, None) == 2
    assert dq(0x10, None, 0, 8, 8, 0x30, None) == 1 and dq(0x10, 0x20, 0, 8, 8, None, None) == 1
    assert dq(0x10, 0x20, 9, 8, 8, 0x30, None) == 5 and dq(0x10, 0x20, 1, -1, 8, 0x30, None) == 2


def test_group_validation(mb):
    """Projection groups: members must agree on T, h, K, dtype and split positions."""
    a, b = _problem(mb), _problem(mb, d=80, ranks=(16, 8))
    g = mb.Group([a, b])
    assert g.validate() == 0
    assert g.workspace_bytes() == a.workspace_bytes() + b.workspace_bytes()
    assert mb.Group([a]).validate() == 0
    assert mb.Group([]).validate() == 2
    assert mb.Group([a] * (mb.MLORA_MAX_GROUP + 1)).validate() == 2
    assert mb.Group([a, _problem(mb, h=64)]).validate() == 2
    assert mb.Group([a, _problem(mb, T=96)]).validate() == 2
    assert mb.Group([a, _problem(mb, off=(0, 16, 64))]).validate() == 3
    assert mb.Group([a, _problem(mb, off=(0, 32, 64, 64), ranks=(8, 4, 4), s=(1.0, 1.0, 1.0))]).validate() == 2
    assert mb.Group([a, _problem(mb, ranks=(8, 200))]).validate() == 4
    c = _problem(mb)
    c.c.dtype = mb.MLORA_F32
    assert mb.Group([a, c]).validate() == 5
    assert mb.Group([a, c]).workspace_bytes() == 0
    assert mb.lib.mlora_lora_group_validate(None, 2) == 1
    # entry points reject before any launch
    ws = g.workspace_bytes()
    two = (ctypes.c_void_p * 2)(0x50, 0x60)
    p2 = ctypes.cast(two, ctypes.POINTER(ctypes.c_void_p))
    hole = (ctypes.c_void_p * 2)(0x50, None)
    ph = ctypes.cast(hole, ctypes.POINTER(ctypes.c_void_p))
    f = mb.lib.mlora_lora_group_fwd
    assert f(g.c, 2, None, p2, p2, 0x40, ws, None) == 1
    assert f(g.c, 2, 0x10, ph, p2, 0x40, ws, None) == 1
    assert f(g.c, 2, 0x10, p2, p2, 0x40, ws - 1, None) == 6
    vpp = ctypes.POINTER(ctypes.c_void_p)
    tab = (vpp * 2)(p2, p2)
    pt = ctypes.cast(tab, ctypes.POINTER(vpp))
    bw = mb.lib.mlora_lora_group_bwd
    assert bw(g.c, 2, 0x10, ph, p2, 0x30, pt, pt, 0, 0x40, ws, None) == 1
    assert bw(g.c, 2, 0x10, p2, p2, 0x30, None, pt, 0, 0x40, ws, None) == 1
    assert bw(g.c, 2, 0x10, p2, p2, 0x30, pt, pt, 0, None, ws, None) == 6


def test_empty_input_is_a_noop(mb):
    p = _problem(mb, T=0, off=(0, 0, 0))
    assert p.validate() == 0
    assert mb.lib.mlora_lora_fwd(ctypes.byref(p.c), None, None, None, None, 0, None) == 0


def test_kernel_path_switch(mb):
    old = mb.set_kernel_path(1)
    assert mb.set_kernel_path(old) == 1


def test_kernel_path_query(mb):
    """A caller can learn, before launching, whether the MFMA kernels or the ~100x slower generic
    kernels will run: bf16, h and d multiples of 64, ranks multiples of 8, 16-byte aligned W, A_k, B_k."""
    fast = _problem(mb, T=64, h=128, d=192, ranks=(8, 16))
    assert fast.kernel_path() == 0
    assert _problem(mb, T=64, h=32, d=48).kernel_path() == 3           # h, d not multiples of 64
    assert _problem(mb, T=64, h=128, d=192, ranks=(8, 4)).kernel_path() == 3  # a rank not a multiple of 8
    odd = _problem(mb, T=64, h=128, d=192, ranks=(8, 16))
    odd.c.W = 0x5008
    assert odd.kernel_path() == 3                                        # misaligned W
    f32 = _problem(mb, T=64, h=128, d=192, ranks=(8, 16))
    f32.c.dtype = mb.MLORA_F32
    assert f32.kernel_path() == 3
    assert _problem(mb, off=(0, 40, 30)).kernel_path() == -1             # invalid problem
    old = mb.set_kernel_path(1)
    try:
        assert fast.kernel_path() == 1
    finally:
        mb.set_kernel_path(old)


def test_workspace_size_does_not_depend_on_addresses(mb):
    """One task of many tokens: the gradient kernels split its tokens over blocks and need
    partial-sum scratch; the size query gives the same answer whatever the pointers are."""
    a = _problem(mb, T=4096, h=256, d=384, off=(0, 4096), ranks=(32,), s=(1.0,))
    b = _problem(mb, T=4096, h=256, d=384, off=(0, 4096), ranks=(32,), s=(1.0,))
    b.c.W = 0x5002
    b._A[0] = 0x2006
    assert a.kernel_path() == 0 and b.kernel_path() == 3
    assert a.workspace_bytes() == b.workspace_bytes() > 4096 * 32 * 2
    assert a.recompute_workspace_bytes() == b.recompute_workspace_bytes()


def test_workloads_match_benchmark_description():
    from paper_2312_02515_amd import workloads as wl
    w = wl.WORKLOADS
    assert w["tiny_f32"].T == 128 and w["tiny_f32"].scalings == [2.0, 2.0]
    assert w["llama2_7b_qproj"].T == 8192
    assert w["llama2_7b_mlp"].T == 16448 and all(t % 64 == 0 and 256 <= t <= 4096 for t in w["llama2_7b_mlp"].tokens)
    assert w["llama2_13b_layer"].T == 32768 and len(w["llama2_13b_layer"].projections) == 7
    assert w["llama2_70b_mlp_stage"].T == 64512 and w["llama2_70b_mlp_stage"].scalings == [2.0] * 32
    total = sum(w["llama2_13b_layer"].flops(p) for p in w["llama2_13b_layer"].projections)
    assert abs(total / 4.22e13 - 1) < 0.01
