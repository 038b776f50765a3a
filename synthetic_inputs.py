"""Seeded synthetic Q/K/V for the spherical-attention workloads.

Shared by the GPU tests, the benchmark and the oracle tests.  It holds no part
of the method's arithmetic: it only draws Gaussian tensors and casts them to
their storage formats.

The paper benchmarks on i.i.d. standard-normal Q, K, V (Section 4.1); the
workloads here keep that distribution with the shapes of the gene-token
sequence configurations.  Recipe, per workload index c:
    generator = torch.Generator('cpu').manual_seed(20250509 + c)
    Q, K, V   = randn([B,H,N,d]) in fp32, drawn in that order
    transform = optional constant factor, then the cast to the storage format
                (bf16, fp16: round-to-nearest-even; e4m3fn: per-tensor factor
                448/max|x|, clamp to +-448, round-to-nearest-even)
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

BASE_SEED = 20250509
E4M3_MAX = 448.0


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    H: int
    N: int
    d: int
    dtype: str          # "f32" | "bf16" | "f16" | "fp8qk_bf16v" | "fp8"
    factor: float = 1.0  # multiplies Q, K and V before the cast

    @property
    def flops(self) -> float:
        """Both contractions: 4*B*H*N^2*d."""
        return 4.0 * self.B * self.H * self.N * self.N * self.d

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def describe(self) -> str:
        return (f"{self.name}: B={self.B} H={self.H} N={self.N} d={self.d} "
                f"{self.dtype} non-causal")


WORKLOADS = {
    "C1": Workload("C1", 0, 1, 1, 256, 64, "f32"),
    "C2": Workload("C2", 1, 4, 8, 2048, 64, "bf16"),
    "C3": Workload("C3", 2, 2, 16, 8192, 128, "bf16"),
    "C4": Workload("C4", 3, 1, 8, 32768, 64, "bf16", factor=1.0 / 8.0),
    "C5": Workload("C5", 4, 4, 16, 16384, 128, "fp8qk_bf16v"),
    # the paper's own benchmark point: FP16, d = 128, N = 3 x 13824 (B and H are not stated)
    "P1": Workload("P1", 5, 1, 8, 41472, 128, "f16"),
}


def gaussian_qkv(B, H, N, d, seed, factor=1.0):
    """Three fp32 CPU tensors [B,H,N,d], i.i.d. N(0,1) times `factor`."""
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    out = []
    for _ in range(3):
        t = torch.randn((B, H, N, d), generator=g, dtype=torch.float32)
        if factor != 1.0:
            t.mul_(factor)
        out.append(t)
    return out


def to_e4m3fn(x: torch.Tensor) -> torch.Tensor:
    """Per-tensor scaled, saturating, round-to-nearest-even cast to OCP E4M3."""
    amax = float(x.abs().max())
    scale = E4M3_MAX / amax if amax > 0 else 1.0
    return (x * scale).clamp_(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn)


def cast_storage(q, k, v, dtype: str):
    """Cast fp32 tensors to the storage formats of `dtype`."""
    if dtype == "f32":
        return q, k, v
    if dtype == "bf16":
        return q.to(torch.bfloat16), k.to(torch.bfloat16), v.to(torch.bfloat16)
    if dtype == "f16":
        return q.to(torch.float16), k.to(torch.float16), v.to(torch.float16)
    if dtype == "fp8qk_bf16v":
        return to_e4m3fn(q), to_e4m3fn(k), v.to(torch.bfloat16)
    if dtype == "fp8":
        return to_e4m3fn(q), to_e4m3fn(k), to_e4m3fn(v)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_qkv(B, H, N, d, dtype, seed, factor=1.0):
    q, k, v = gaussian_qkv(B, H, N, d, seed, factor)
    return cast_storage(q, k, v, dtype)


def make_workload(name: str):
    """A named workload, or a shape of one's own written "B,H,N,d" or "B,H,N,d,dtype" (bf16
    when not given; seed BASE_SEED + 99)."""
    if "," in name:
        parts = name.split(",")
        B, H, N, d = (int(x) for x in parts[:4])
        w = Workload(name, 99, B, H, N, d, parts[4] if len(parts) > 4 else "bf16")
    else:
        w = WORKLOADS[name]
    return w, make_qkv(w.B, w.H, w.N, w.d, w.dtype, w.seed, w.factor)


def storage_bits(t: torch.Tensor):
    """(numpy array, kind) in the form the oracle accepts, sharing memory with `t`."""
    t = t.contiguous()
    if t.dtype == torch.float32:
        return t.numpy(), "f32"
    if t.dtype == torch.float64:
        return t.numpy(), "f64"
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16), "bf16"
    if t.dtype == torch.float16:
        return t.view(torch.int16).numpy().view(np.uint16), "f16"
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy(), "e4m3fn"
    raise TypeError(f"unsupported storage dtype {t.dtype}")
