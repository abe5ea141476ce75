"""Seeded synthetic LRM-shaped inputs.

This module only draws random tensors and rounds them to bf16 with the
library cast.  It holds none of the method's arithmetic (no amax, scale,
FP8 cast, GEMM, norm or probe code), so both the CPU oracle's tests and the
HIP path's tests may draw their operands from it.

The paper's layers are production recommendation-model linears whose inputs
are described as heavy-tailed with systematic outlier channels (Section 2.3,
"Characterizing Low-Precision Quantization Overheads and Error in LRMs");
none of that data is public, so each workload below is a synthetic stand-in
with the stated shape and value distribution.

All tensors are CPU torch.bfloat16, row-major.  X is [M, K], W is [K, N].
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    N: int
    batch: int          # number of independent (X, W) problems (grouped launch)
    x_dist: str         # "normal" | "student_t4" | "normal_outlier4"
    norm: str           # "layernorm" | "rmsnorm"
    seed: int
    eps: float = 1e-5


WORKLOADS = {
    # single FP8 linear + LayerNorm, launch-latency sized
    "C1": Workload("C1", 256, 128, 128, 1, "normal", "layernorm", 0),
    # LRM MLP layer, heavy tails, RMSNorm epilogue
    "C2": Workload("C2", 16384, 512, 512, 1, "student_t4", "rmsnorm", 1),
    # skinny pair (layer a feeds layer b through its LayerNorm output)
    "C3a": Workload("C3a", 65536, 256, 1024, 1, "normal", "layernorm", 2),
    "C3b": Workload("C3b", 65536, 1024, 256, 1, "normal", "layernorm", 3),
    # 64 grouped small GEMMs with a fused RMSNorm per group
    "C4": Workload("C4", 4096, 256, 256, 64, "normal", "rmsnorm", 1000),
    # outlier-heavy large layer
    "C5": Workload("C5", 32768, 4096, 4096, 1, "normal_outlier4", "layernorm", 4),
}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def normal(rows: int, cols: int, seed: int, std: float = 1.0) -> torch.Tensor:
    """[rows, cols] bf16 ~ N(0, std^2)."""
    x = torch.randn(rows, cols, generator=_gen(seed), dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    return x.to(torch.bfloat16)


def student_t4(rows: int, cols: int, seed: int) -> torch.Tensor:
    """[rows, cols] bf16 ~ Student-t(nu=4) scaled to unit variance (heavy tails).

    t = Z / sqrt(chi2_4 / 4) has variance nu/(nu-2) = 2, so it is divided by sqrt(2).
    """
    g = _gen(seed)
    z = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    chi = torch.zeros(rows, cols, dtype=torch.float32)
    for _ in range(4):
        c = torch.randn(rows, cols, generator=g, dtype=torch.float32)
        chi.addcmul_(c, c)
    z.div_(torch.sqrt(chi.div_(4.0))).div_(math.sqrt(2.0))
    return z.to(torch.bfloat16)


def normal_outlier4(rows: int, cols: int, seed: int, factor: float = 100.0):
    """[rows, cols] bf16 ~ N(0,1) with 4 seeded random channels (columns) scaled by `factor`.

    Returns (x, outlier_columns).
    """
    g = _gen(seed)
    x = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    cols_idx = torch.randperm(cols, generator=g)[:4].sort().values
    x[:, cols_idx] *= factor
    return x.to(torch.bfloat16), cols_idx


def correlated(rows: int, cols: int, seed: int, mean_span: float = 2.0, mix: float = 0.6) -> torch.Tensor:
    """[rows, cols] bf16 with a non-zero per-column mean and correlated columns: x = 1 mu^T + Z L^T with a
    banded lower-triangular L (each column mixes `mix` of its left neighbour's noise) and mu ~ U(-span, span).
    Stands in for a layer input whose distribution the online tracker learns (means of the size of the
    standard deviations, so the mean correction of the scatter matters)."""
    g = _gen(seed)
    z = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    mu = (torch.rand(cols, generator=g, dtype=torch.float32) * 2.0 - 1.0) * mean_span
    sd = 0.25 + 1.5 * torch.rand(cols, generator=g, dtype=torch.float32)
    x = z.clone()
    x[:, 1:] += mix * z[:, :-1]
    return (x * sd + mu).to(torch.bfloat16)


def weight(K: int, N: int, seed: int) -> torch.Tensor:
    """[K, N] bf16 ~ N(0, 1/K)."""
    return normal(K, N, seed, std=1.0 / math.sqrt(K))


def activations(w: Workload, group: int = 0, rows: int | None = None) -> torch.Tensor:
    """X for workload `w` (group `group` of a grouped workload).

    `rows` < M draws only that many rows; because the generator is sequential
    the first `rows` rows of the "normal" distribution equal those of the full
    draw, but this is not relied on anywhere: a reduced draw is simply a
    smaller workload of the same distribution.
    """
    M = w.M if rows is None else rows
    seed = w.seed + group
    if w.x_dist == "normal":
        return normal(M, w.K, seed)
    if w.x_dist == "student_t4":
        return student_t4(M, w.K, seed)
    if w.x_dist == "normal_outlier4":
        return normal_outlier4(M, w.K, seed)[0]
    raise ValueError(w.x_dist)


def weights(w: Workload, group: int = 0) -> torch.Tensor:
    return weight(w.K, w.N, 7919 * (w.seed + group) + 13)


def affine(N: int, seed: int):
    """Non-trivial LayerNorm/RMSNorm gamma, beta (bf16 [N]) for tests that exercise them."""
    g = _gen(seed)
    gamma = (1.0 + 0.25 * torch.randn(N, generator=g)).to(torch.bfloat16)
    beta = (0.1 * torch.randn(N, generator=g)).to(torch.bfloat16)
    return gamma, beta


def bf16_bits(t: torch.Tensor):
    """View a bf16 CPU tensor as a numpy uint16 array (no copy)."""
    import numpy as np

    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a) -> torch.Tensor:
    """Inverse of bf16_bits."""
    import numpy as np

    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
