"""Seeded synthetic inputs for the fused residual-add + RMSNorm workloads.

This module holds no arithmetic of the operator: it draws numbers and casts
them to the storage format, nothing else.  The same tensors feed the GPU
library and whatever they are checked against, so both see identical bits.

Recipe (one torch CPU generator per workload, seeded with ``seed``; draws are
made in the fixed order x, residual, weight, [outlier mask, outlier values];
everything is drawn in fp32 and cast round-to-nearest-even to storage):

    x        ~ N(0, x_std)       second argument is a standard deviation
    residual ~ N(0, r_std)
    weight   ~ U(w_lo, w_hi)
    outliers : each x entry is replaced, with probability ``outlier_p``
               (independent Bernoulli per element), by a draw from
               N(0, outlier_std)

The shapes stand in for LLM activations entering a norm layer: ``M`` tokens
(prefill: thousands; decode: 1..256) by a hidden size ``N``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np
import torch

DTYPES = ("bf16", "fp16", "fp16_res32", "fp32")


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    dtype: str
    eps: float
    seed: int
    x_std: float = 1.0
    r_std: float = 1.0
    w_lo: float = 0.5
    w_hi: float = 1.5
    outlier_p: float = 0.0
    outlier_std: float = 0.0

    def with_rows(self, M: int) -> "Workload":
        return replace(self, M=M, name=f"{self.name}[M={M}]")

    def with_cols(self, N: int) -> "Workload":
        return replace(self, N=N, name=f"{self.name}[N={N}]")


# The five benchmark configurations.
SMOKE = Workload("smoke_16x4096_bf16", 16, 4096, "bf16", 1e-6, 0)
PREFILL = Workload("prefill_4096x4096_bf16", 4096, 4096, "bf16", 1e-6, 1)
DECODE = Workload("decode_Mx8192_bf16", 256, 8192, "bf16", 1e-5, 2, x_std=2.0, r_std=2.0)
DECODE_M = (1, 2, 4, 8, 16, 32, 64, 128, 256)
LARGE_PREFILL = Workload("large_prefill_32768x7168_bf16_outliers", 32768, 7168, "bf16", 1e-6, 3,
                         outlier_p=0.01, outlier_std=50.0)
ODD_WIDTH = Workload("odd_width_8192xN_fp16_res32", 8192, 5120, "fp16_res32", 1e-6, 4,
                     w_lo=0.8, w_hi=1.2)
ODD_WIDTH_N = (5120, 2880, 1000)

CONFIGS: Dict[str, Workload] = {
    "smoke": SMOKE, "prefill": PREFILL, "decode": DECODE,
    "large_prefill": LARGE_PREFILL, "odd_width": ODD_WIDTH,
}


def x_torch_dtype(dtype: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp16": torch.float16,
            "fp16_res32": torch.float16, "fp32": torch.float32}[dtype]


def r_torch_dtype(dtype: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp16": torch.float16,
            "fp16_res32": torch.float32, "fp32": torch.float32}[dtype]


def x_bytes(dtype: str) -> int:
    return 4 if dtype == "fp32" else 2


def r_bytes(dtype: str) -> int:
    return 4 if dtype in ("fp32", "fp16_res32") else 2


def algorithmic_bytes(M: int, N: int, dtype: str) -> int:
    """Bytes the operator must move: x and residual read once and written once,
    the weight vector read once."""
    return M * N * (2 * x_bytes(dtype) + 2 * r_bytes(dtype)) + N * x_bytes(dtype)


def generate(wl: Workload) -> Dict[str, torch.Tensor]:
    """CPU tensors ``x`` [M,N], ``r`` [M,N], ``w`` [N] in storage dtype."""
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed)
    shape = (wl.M, wl.N)
    x = torch.randn(shape, generator=g, dtype=torch.float32) * wl.x_std
    r = torch.randn(shape, generator=g, dtype=torch.float32) * wl.r_std
    w = torch.rand((wl.N,), generator=g, dtype=torch.float32) * (wl.w_hi - wl.w_lo) + wl.w_lo
    if wl.outlier_p > 0.0:
        mask = torch.rand(shape, generator=g, dtype=torch.float32) < wl.outlier_p
        out = torch.randn(shape, generator=g, dtype=torch.float32) * wl.outlier_std
        x = torch.where(mask, out, x)
        del mask, out
    return {
        "x": x.to(x_torch_dtype(wl.dtype)).contiguous(),
        "r": r.to(r_torch_dtype(wl.dtype)).contiguous(),
        "w": w.to(x_torch_dtype(wl.dtype)).contiguous(),
    }


def to_bits(t: torch.Tensor) -> np.ndarray:
    """View a CPU tensor as the array type used for bit comparison: uint16 bit
    patterns for bf16/fp16, float32 as is."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


# ---- silu_and_mul -----------------------------------------------------------------------

@dataclass(frozen=True)
class GatedWorkload:
    """Input of the gated activation: x [M, 2d] ~ N(0, x_std), gate half first then up half.
    d stands in for the feed-forward width of an LLM layer (11008, 13824, 14336, 28672)."""
    name: str
    M: int
    d: int
    dtype: str
    seed: int
    x_std: float = 1.5


SILU_PREFILL = GatedWorkload("silu_prefill_4096x11008_bf16", 4096, 11008, "bf16", 11)
SILU_DECODE = GatedWorkload("silu_decode_64x14336_bf16", 64, 14336, "bf16", 12)
SILU_FP16 = GatedWorkload("silu_2048x13824_fp16", 2048, 13824, "fp16", 13)


def silumul_algorithmic_bytes(M: int, d: int, dtype: str) -> int:
    """Both halves of x read once, out written once."""
    return 3 * M * d * x_bytes(dtype)


def generate_gated(wl: GatedWorkload) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed)
    x = torch.randn((wl.M, 2 * wl.d), generator=g, dtype=torch.float32) * wl.x_std
    return x.to(x_torch_dtype(wl.dtype)).contiguous()


# ---- merge_attn_states --------------------------------------------------------------------

@dataclass(frozen=True)
class MergeWorkload:
    """Two partial attention states to merge: v_a, v_b [n*h, d] ~ N(0, 1) in storage dtype and
    their log-sum-exp scores s_a, s_b [n*h] ~ N(0, s_std) in fp32.  (n, h, d) stands for
    tokens x heads x head size; the tuples below are of the kind the paper lists for its
    3-D shaped kernel (Section 4, Kernels)."""
    name: str
    n: int
    h: int
    d: int
    dtype: str
    seed: int
    s_std: float = 3.0

    @property
    def rows(self) -> int:
        return self.n * self.h


MERGE_SHAPES = ((512, 32, 256), (512, 40, 128), (768, 32, 256), (768, 40, 128), (512, 64, 128))
MERGE_MAIN = MergeWorkload("merge_512x32x256_bf16", 512, 32, 256, "bf16", 21)


def merge_algorithmic_bytes(rows: int, d: int, dtype: str) -> int:
    return rows * (3 * d * x_bytes(dtype) + 12)


def generate_merge(wl: MergeWorkload) -> Dict[str, torch.Tensor]:
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed)
    shape = (wl.rows, wl.d)
    va = torch.randn(shape, generator=g, dtype=torch.float32)
    vb = torch.randn(shape, generator=g, dtype=torch.float32)
    sa = torch.randn((wl.rows,), generator=g, dtype=torch.float32) * wl.s_std
    sb = torch.randn((wl.rows,), generator=g, dtype=torch.float32) * wl.s_std
    dt = x_torch_dtype(wl.dtype)
    return {"va": va.to(dt).contiguous(), "vb": vb.to(dt).contiguous(), "sa": sa.contiguous(), "sb": sb.contiguous()}
