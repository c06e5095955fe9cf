"""Seeded synthetic inputs for the attention forward pass.

This module only draws random tensors; it holds none of the method's arithmetic, so both the
GPU tests/benchmark and the CPU oracle's tests may use it.  The five workloads are the ones the
benchmark definition lists (shapes chosen so that the K+V bytes of one head are 0.06, 0.5, 4, 8
and 16 MiB, i.e. below, at and above one XCD's 4 MiB L2).  The paper's own workloads are shape
sweeps with unstated values (Sec. 3.1, Sec. 4.2, Sec. 4.3), so values are i.i.d. normal.

Recipe (identical on every machine: the CPU generator is used, never the device one):
    g = torch.Generator('cpu').manual_seed(seed)
    Q, K, V = randn(B,H,N,d) drawn in that order in fp32, multiplied by `gain` in fp32,
    workload 5 only: one offset vector per (batch, head), randn(B,H,1,d) * 0.5, drawn after V and
    added to every K row in fp32;  then one cast to the storage dtype.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    causal: bool
    dtype: str          # "f16" | "bf16"
    seed: int
    gain: float = 1.0
    k_offset_std: float = 0.0

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def flops(self) -> float:
        """4*B*H*N^2*d (two contractions, 2 flops per multiply-add), halved under a causal mask."""
        f = 4.0 * self.B * self.H * float(self.N) * float(self.N) * self.d
        return f / 2 if self.causal else f

    @property
    def torch_dtype(self):
        return {"f16": torch.float16, "bf16": torch.bfloat16}[self.dtype]


WORKLOADS = {
    1: Workload("cfg1_B1_H1_N256_d64_f16", 1, 1, 256, 64, False, "f16", 0),
    2: Workload("cfg2_B1_H8_N2048_d64_f16", 1, 8, 2048, 64, False, "f16", 1),
    3: Workload("cfg3_B1_H16_N8192_d128_bf16_causal", 1, 16, 8192, 128, True, "bf16", 2),
    4: Workload("cfg4_B1_H32_N16384_d128_f16", 1, 32, 16384, 128, False, "f16", 3, gain=0.5),
    5: Workload("cfg5_B4_H32_N32768_d128_bf16_causal", 4, 32, 32768, 128, True, "bf16", 4,
                k_offset_std=0.5),
}


def make_qkv(w: Workload, device: str = "cpu"):
    """Draw (Q, K, V) for a workload; tensors are [B, H, N, d] contiguous in the storage dtype."""
    g = torch.Generator("cpu").manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.d)
    out = []
    k32 = None
    for name in ("Q", "K", "V"):
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        if w.gain != 1.0:
            x.mul_(w.gain)
        if name == "K" and w.k_offset_std != 0.0:
            k32 = x           # the offset is drawn after V; the cast of K waits for it
            out.append(None)
            continue
        out.append(x.to(w.torch_dtype))
        del x
    if k32 is not None:
        off = torch.randn((w.B, w.H, 1, w.d), generator=g, dtype=torch.float32) * w.k_offset_std
        k32.add_(off)
        out[1] = k32.to(w.torch_dtype)
        del k32
    if device != "cpu":
        out = [t.to(device) for t in out]
    return tuple(out)


def make_random(B: int, H: int, N: int, d: int, dtype: str, seed: int, gain: float = 1.0,
                device: str = "cpu"):
    """Free-form i.i.d. normal inputs for shapes outside the five workloads (ragged N, tiny N)."""
    w = Workload(f"rand_B{B}_H{H}_N{N}_d{d}_{dtype}", B, H, N, d, False, dtype, seed, gain=gain)
    return make_qkv(w, device)
