"""Workload shapes and seeded synthetic input generators.

This module holds NO arithmetic of the method: it only names the five benchmark
configurations (shapes, segment lengths, ranks, scalings) and draws random
tensors.  Both the CPU oracle's tests and the HIP path's tests/benchmark obtain
their inputs here, so both sides consume the same bit patterns; the oracle
widens them to float64, the HIP path reads them as stored.

Stand-in statement: the paper measures on GSM8K with Llama-2 / TinyLlama
weights (section 4.1).  Neither is available here; the cost of the operator
depends on shapes, segment lengths and ranks only, so seeded random tensors of
Llama-2 layer shapes stand in for them.

Value distributions (all configurations):
  X  ~ N(0,1)            dY ~ N(0,1)
  W  ~ N(0, sigma_w^2)   sigma_w = 1/16 for the tiny case, 0.02 otherwise
  A_k ~ U(-1/sqrt(h), 1/sqrt(h))   (Kaiming-uniform, a = sqrt(5), fan-in h)
  B_k ~ N(0, 0.02^2)     (non-zero on purpose so that dA_k != 0)
  alpha_k = 2 r_k  =>  s_k = 2.0
Values are drawn in float32 with a seeded torch generator on the device asked
for and then rounded to the configuration's storage dtype.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Sequence, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class Projection:
    name: str
    h: int  # input features  (rows of W)
    d: int  # output features (columns of W)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16"
    tokens: Tuple[int, ...]         # t_k per adapter
    ranks: Tuple[int, ...]          # r_k per adapter
    alphas: Tuple[float, ...]       # alpha_k per adapter
    projections: Tuple[Projection, ...]
    sigma_w: float

    @property
    def K(self) -> int:
        return len(self.tokens)

    @property
    def T(self) -> int:
        return int(sum(self.tokens))

    @property
    def seg_offsets(self) -> List[int]:
        off = [0]
        for t in self.tokens:
            off.append(off[-1] + int(t))
        return off

    @property
    def scalings(self) -> List[float]:
        return [float(a) / float(r) for a, r in zip(self.alphas, self.ranks)]

    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def flops(self, proj: Projection) -> float:
        """Useful flops of forward + backward of one projection:
        4 T h d + 6 sum_k t_k r_k (h + d)."""
        f = 4.0 * self.T * proj.h * proj.d
        for t, r in zip(self.tokens, self.ranks):
            f += 6.0 * t * r * (proj.h + proj.d)
        return f


_CFG3_TOKENS = (3392, 576, 896, 1152, 960, 3328, 3648, 2496)
_CFG5_TOKENS = (512, 512, 4096, 1024, 2048, 2048, 2048, 512, 1024, 512, 1024, 4096,
                2048, 512, 2048, 512, 4096, 4096, 4096, 2048, 4096, 1024, 512, 2048,
                1024, 2048, 4096, 1024, 4096, 512, 1024, 4096)


def _mk(name, dtype, tokens, ranks, projections, sigma_w):
    return Workload(name=name, dtype=dtype, tokens=tuple(tokens), ranks=tuple(ranks),
                    alphas=tuple(2.0 * r for r in ranks),
                    projections=tuple(Projection(*p) for p in projections), sigma_w=sigma_w)


WORKLOADS = {
    "tiny_f32": _mk("tiny_f32", "f32", (64, 64), (8, 8), [("w", 256, 256)], 1.0 / 16.0),
    "llama2_7b_qproj": _mk("llama2_7b_qproj", "bf16", (2048,) * 4, (16,) * 4,
                           [("q_proj", 4096, 4096)], 0.02),
    "llama2_7b_mlp": _mk("llama2_7b_mlp", "bf16", _CFG3_TOKENS, (8, 16, 32, 64) * 2,
                         [("gate_proj", 4096, 11008), ("up_proj", 4096, 11008),
                          ("down_proj", 11008, 4096)], 0.02),
    "llama2_13b_layer": _mk("llama2_13b_layer", "bf16", (2048,) * 16, (8, 16, 32, 64) * 4,
                            [("q_proj", 5120, 5120), ("k_proj", 5120, 5120),
                             ("v_proj", 5120, 5120), ("o_proj", 5120, 5120),
                             ("gate_proj", 5120, 13824), ("up_proj", 5120, 13824),
                             ("down_proj", 13824, 5120)], 0.02),
    "llama2_70b_mlp_stage": _mk("llama2_70b_mlp_stage", "bf16", _CFG5_TOKENS, (64,) * 32,
                                [("up_proj", 8192, 28672), ("down_proj", 28672, 8192)], 0.02),
}

# order in which the benchmark description lists them (index 0 = tiny case)
WORKLOAD_ORDER = ["tiny_f32", "llama2_7b_qproj", "llama2_7b_mlp", "llama2_13b_layer",
                  "llama2_70b_mlp_stage"]


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _sub_seed(seed: int, *ids: int) -> int:
    """Mix a few small integers into one 63-bit seed (splitmix-style)."""
    x = (int(seed) * 0x9E3779B97F4A7C15 + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF
    for i in ids:
        x ^= (int(i) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2)) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def normal(shape: Sequence[int], std: float, dtype: torch.dtype, device, seed: int) -> torch.Tensor:
    g = _gen(device, seed)
    n = 1
    for s_ in shape:
        n *= int(s_)
    if n >= (1 << 28):
        # large tensors: draw in the storage dtype slab by slab to bound the fp32 temporary
        out = torch.empty(tuple(shape), dtype=dtype, device=device)
        flat = out.view(-1)
        step = 1 << 27
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            flat[lo:hi] = (torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
        return out
    return (torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32) * std).to(dtype)


def uniform(shape: Sequence[int], bound: float, dtype: torch.dtype, device, seed: int) -> torch.Tensor:
    g = _gen(device, seed)
    u = torch.rand(tuple(shape), generator=g, device=device, dtype=torch.float32)
    return ((u * 2.0 - 1.0) * bound).to(dtype)


@dataclasses.dataclass
class Inputs:
    X: torch.Tensor                 # [T,h]
    W: torch.Tensor                 # [h,d]
    dY: torch.Tensor                # [T,d]
    A: List[torch.Tensor]           # [h,r_k]
    B: List[torch.Tensor]           # [r_k,d]
    seg_offsets: List[int]
    ranks: List[int]
    scalings: List[float]


def make_inputs(T: int, h: int, d: int, seg_offsets: Sequence[int], ranks: Sequence[int],
                scalings: Sequence[float], dtype: torch.dtype, device="cpu", seed: int = 0,
                sigma_w: float = 0.02, proj_id: int = 0) -> Inputs:
    """Draw one problem instance.  Tensor ids: 1=X 2=W 3=dY 4=A_k 5=B_k."""
    X = normal((T, h), 1.0, dtype, device, _sub_seed(seed, proj_id, 1))
    W = normal((h, d), sigma_w, dtype, device, _sub_seed(seed, proj_id, 2))
    dY = normal((T, d), 1.0, dtype, device, _sub_seed(seed, proj_id, 3))
    A, B = [], []
    for k, r in enumerate(ranks):
        A.append(uniform((h, r), 1.0 / math.sqrt(h), dtype, device, _sub_seed(seed, proj_id, 4, k)))
        B.append(normal((r, d), 0.02, dtype, device, _sub_seed(seed, proj_id, 5, k)))
    return Inputs(X=X, W=W, dY=dY, A=A, B=B, seg_offsets=list(int(o) for o in seg_offsets),
                  ranks=list(int(r) for r in ranks), scalings=list(float(s) for s in scalings))


def make_workload_inputs(wl: Workload, proj_index: int, device="cpu", seed: int = 0) -> Inputs:
    p = wl.projections[proj_index]
    return make_inputs(wl.T, p.h, p.d, wl.seg_offsets, wl.ranks, wl.scalings, wl.torch_dtype(),
                       device=device, seed=seed, sigma_w=wl.sigma_w, proj_id=proj_index)


def sample_rows(seg_offsets: Sequence[int], T: int, per_adapter: int, seed: int, tile: int = 256) -> List[int]:
    """Rows for sampled checks: for each non-empty segment its first and last row
    and `per_adapter` seeded draws; the rows on both sides of every segment
    boundary; one row from each uncovered range; and, so that no output tile of
    `tile` rows goes unchecked, the first row, the last row and one seeded draw
    of every such tile (tile = 0 leaves these out)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    rows = set()
    K = len(seg_offsets) - 1
    for k in range(K):
        lo, hi = int(seg_offsets[k]), int(seg_offsets[k + 1])
        if hi <= lo:
            continue
        rows.update((lo, hi - 1))
        draws = torch.randint(lo, hi, (per_adapter,), generator=g)
        rows.update(int(v) for v in draws)
    for o in seg_offsets:
        for r in (int(o) - 1, int(o)):
            if 0 <= r < T:
                rows.add(r)
    if K >= 0 and int(seg_offsets[0]) > 0:
        rows.add(0)
    if int(seg_offsets[-1]) < T:
        rows.add(T - 1)
    if tile > 0 and T > 0:
        n_tiles = (T + tile - 1) // tile
        draws = torch.randint(0, tile, (n_tiles,), generator=g)
        for i in range(n_tiles):
            lo, hi = i * tile, min(T, (i + 1) * tile)
            rows.update((lo, hi - 1, min(lo + int(draws[i]), hi - 1)))
    return sorted(rows)
