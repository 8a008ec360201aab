"""Seeded synthetic weight tensors for the five benchmark workloads.

This module holds input generation only -- none of the quantization method's
arithmetic -- so that both the HIP path and the CPU oracle can be fed from it
without sharing any code of the method.  The tensors stand in for LLM linear
layer weights (heavy-tailed entries plus a few large input-channel columns).

Every tensor is drawn in float32 from a ``torch.Generator`` seeded with
``1000 * workload + tensor_index`` on the requested device and rounded to bf16
(round to nearest even).  A tensor generated on the GPU is copied to the host
for the oracle; the two sides never need to agree on a random stream.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Iterator, List, Optional

import torch


@dataclass(frozen=True)
class TensorSpec:
    workload: int          # 1..5
    index: int             # position inside the workload
    name: str
    rows: int
    cols: int
    dss_radius: int        # K: candidates are the E4M3 codes centre-K .. centre+K
    dist: str              # "normal" | "t"
    df: int                # Student-t degrees of freedom (dist == "t")
    std: float             # target standard deviation of the bulk
    entry_outlier_p: float = 0.0      # Bernoulli rate of entry-level outliers
    entry_outlier_mode: str = ""      # "replace_t3" | "mul"
    entry_outlier_scale: float = 1.0
    n_outlier_cols: int = 0
    col_scale_lo: float = 1.0
    col_scale_hi: float = 1.0

    @property
    def seed(self) -> int:
        return 1000 * self.workload + self.index

    @property
    def numel(self) -> int:
        return self.rows * self.cols


def _student_t(shape, df: int, gen: torch.Generator, device) -> torch.Tensor:
    """t_df = z / sqrt(chi2_df / df), chi2_df as a sum of df squared normals."""
    z = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(df):
        g = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        chi2.addcmul_(g, g)
        del g
    chi2.div_(df).sqrt_()
    z.div_(chi2)
    return z


def make_weight(spec: TensorSpec, device="cpu", dtype=torch.bfloat16,
                std_override: Optional[float] = None) -> torch.Tensor:
    """Draw the tensor described by ``spec`` (bf16 by default, float32 on request)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(spec.seed)
    shape = (spec.rows, spec.cols)
    std = spec.std if std_override is None else std_override
    if spec.dist == "normal":
        w = torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * std
    elif spec.dist == "t":
        w = _student_t(shape, spec.df, gen, device)
        # Var t_df = df / (df - 2): rescale to the target standard deviation
        w.mul_(std / math.sqrt(spec.df / (spec.df - 2.0)))
    else:
        raise ValueError(spec.dist)
    if spec.entry_outlier_p > 0.0:
        mask = torch.rand(shape, generator=gen, device=device) < spec.entry_outlier_p
        if spec.entry_outlier_mode == "replace_t3":
            t3 = _student_t(shape, 3, gen, device) * spec.entry_outlier_scale
            w = torch.where(mask, t3, w)
            del t3
        elif spec.entry_outlier_mode == "mul":
            w = torch.where(mask, w * spec.entry_outlier_scale, w)
        else:
            raise ValueError(spec.entry_outlier_mode)
        del mask
    if spec.n_outlier_cols > 0:
        cols = torch.randperm(spec.cols, generator=gen, device=device)[: spec.n_outlier_cols]
        if spec.col_scale_hi > spec.col_scale_lo:
            u = torch.rand(spec.n_outlier_cols, generator=gen, device=device)
            f = spec.col_scale_lo + (spec.col_scale_hi - spec.col_scale_lo) * u
        else:
            f = torch.full((spec.n_outlier_cols,), spec.col_scale_lo, device=device)
        w[:, cols] *= f.to(torch.float32)[None, :]
    return w.to(dtype).contiguous()


def _layer_std_jitter(workload: int, layer: int) -> float:
    """Per-layer standard deviation 0.02 * U(0.7, 1.3), from a seed of its own."""
    g = torch.Generator(device="cpu")
    g.manual_seed(900_000 + 1000 * workload + layer)
    return 0.02 * (0.7 + 0.6 * float(torch.rand((), generator=g)))


def workload_specs(workload: int, scale_down: int = 1) -> List[TensorSpec]:
    """Tensor list of workload 1..5.

    ``scale_down`` divides every dimension (kept a multiple of 16) so that the
    same recipe can be exercised at sizes a CPU finishes in seconds.
    """
    def d(n: int) -> int:
        return max(16, (n // scale_down) // 16 * 16)

    if workload == 1:
        return [TensorSpec(1, 0, "w", d(256), d(256), 4, "normal", 0, 0.02,
                           entry_outlier_p=0.01, entry_outlier_mode="replace_t3",
                           entry_outlier_scale=0.2)]
    if workload == 2:
        return [TensorSpec(2, 0, "attn_proj", d(4096), d(4096), 4, "t", 4, 0.02,
                           n_outlier_cols=8, col_scale_lo=20.0, col_scale_hi=20.0)]
    if workload == 3:
        cols = d(4096)
        return [TensorSpec(3, 0, "mlp_up", d(14336), cols, 8, "t", 4, 0.02,
                           n_outlier_cols=max(1, round(0.005 * cols)),
                           col_scale_lo=10.0, col_scale_hi=50.0)]
    if workload == 4:
        shapes = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                  ("gate", 12288, 4096), ("up", 12288, 4096), ("down", 4096, 12288)]
        out = []
        for layer in range(36):
            std = _layer_std_jitter(4, layer)
            for k, (nm, r, c) in enumerate(shapes):
                out.append(TensorSpec(4, layer * 7 + k, f"L{layer}.{nm}", d(r), d(c), 4, "t", 4, std,
                                      n_outlier_cols=16, col_scale_lo=20.0, col_scale_hi=20.0))
        return out
    if workload == 5:
        shapes = [("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]
        out = []
        for layer in range(80):
            for k, (nm, r, c) in enumerate(shapes):
                out.append(TensorSpec(5, layer * 3 + k, f"L{layer}.{nm}", d(r), d(c), 8, "t", 3, 0.015,
                                      entry_outlier_p=0.001, entry_outlier_mode="mul",
                                      entry_outlier_scale=50.0,
                                      n_outlier_cols=32, col_scale_lo=30.0, col_scale_hi=30.0))
        return out
    raise ValueError("workload must be 1..5")


def iter_workload(workload: int, device="cpu", scale_down: int = 1) -> Iterator:
    for spec in workload_specs(workload, scale_down):
        yield spec, make_weight(spec, device)


def bf16_bits(t: torch.Tensor):
    """uint16 numpy view of a bf16 CPU tensor (what the oracle's ctypes layer takes)."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view("uint16")
