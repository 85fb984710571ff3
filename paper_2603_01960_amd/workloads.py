"""Seeded synthetic workloads (shapes, dtypes, value distributions).

This module only draws random tensors; it contains none of the attention
arithmetic and is the one module that both the device tests and the CPU-side
checks may use.  The paper benchmarks random tensors with identical
initialisation across methods (Section 4.3); its "text" and "vision" regimes
are shape regimes (D = 64 / 128, S from hundreds to thousands), so seeded
normal tensors of those shapes are the workload itself.

Recipe: ``g = torch.Generator('cpu').manual_seed(seed)``; draw float32 standard
normals of shape [B, H, S, D] in the order Q, K, V; multiply by the per-tensor
standard deviation; cast once (round-to-nearest-even) to FP16 or BF16.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    S: int
    D: int
    dtypes: Tuple[str, ...]          # "f16" / "bf16"
    seed: int
    qk_std: float = 1.0              # standard deviation of Q and K entries
    v_std: float = 1.0
    note: str = ""

    @property
    def BH(self) -> int:
        return self.B * self.H

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def flops(self) -> float:
        """4*B*H*S^2*D: the two matrix products of the non-causal forward pass."""
        return 4.0 * self.B * self.H * self.S * self.S * self.D

    def compulsory_bytes(self, bytes_per_elem: int = 2) -> float:
        """Q, K, V read once and O written once (the paper's bandwidth-proxy numerator, Eq. 7)."""
        return 4.0 * self.B * self.H * self.S * self.D * bytes_per_elem


# N(0,2) is read as mean 0, variance 2 (standard deviation sqrt(2)).
WORKLOADS = {
    "C1": Workload("C1", 1, 2, 128, 64, ("f16",), 1001, note="small case"),
    "C2": Workload("C2", 4, 16, 1024, 64, ("f16", "bf16"), 1002, note="text regime"),
    "C3": Workload("C3", 64, 12, 197, 64, ("bf16",), 1003, note="vision regime, ragged S"),
    "C4": Workload("C4", 2, 32, 8192, 128, ("bf16",), 1004, note="long context"),
    "C5": Workload("C5", 1, 16, 16384, 128, ("f16",), 1005, qk_std=math.sqrt(2.0),
                   note="long context, peaked softmax"),
}

TORCH_DTYPES = {"f16": torch.float16, "bf16": torch.bfloat16}


def make_qkv(B: int, H: int, S: int, D: int, dtype: str, seed: int,
             qk_std: float = 1.0, v_std: float = 1.0):
    """Return CPU tensors (q, k, v), each [B, H, S, D] in the requested 16-bit dtype."""
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    tdt = TORCH_DTYPES[dtype]
    out = []
    for std in (qk_std, qk_std, v_std):
        x = torch.randn(B, H, S, D, dtype=torch.float32, generator=g)
        if std != 1.0:
            x = x * float(std)
        out.append(x.to(tdt).contiguous())
    return tuple(out)


def make_workload(name: str, dtype: str | None = None):
    """Return (workload, q, k, v) for one of the named configurations."""
    w = WORKLOADS[name]
    dt = dtype or w.dtypes[0]
    if dt not in TORCH_DTYPES:
        raise ValueError(f"unknown dtype {dt}")
    q, k, v = make_qkv(w.B, w.H, w.S, w.D, dt, w.seed, w.qk_std, w.v_std)
    return w, q, k, v


def sample_rows(S: int, tile_sizes=(32, 64, 128), stride: int = 509, limit: int | None = None):
    """Query rows for sampled parity at large S: first, last, both sides of EVERY multiple of each
    tile size (32 = the rows of one wavefront, 64 and 128 = the query tiles), and a fixed stride
    through the rest.  ``limit`` thins only the stride rows; boundary rows are always all kept."""
    edge = {0, S - 1}
    for t in tile_sizes:
        for b in range(t, S, t):
            edge.add(b - 1)
            edge.add(b)
    extra = sorted(set(range(0, S, stride)) - edge)
    if limit is not None and len(extra) > limit:
        step = len(extra) / float(max(limit, 1))
        extra = [extra[int(i * step)] for i in range(max(limit, 0))]
    return sorted(r for r in edge.union(extra) if 0 <= r < S)
