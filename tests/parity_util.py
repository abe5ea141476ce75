"""Helpers shared by the GPU parity tests: tolerances and oracle drivers.

Tolerances (each derived from the arithmetic it bounds):
 * codes, scales, rowmax: bit-exact.
 * fp32 Y: the gfx950 FP8 MFMA aligns the eight products of each group of 8 consecutive
   K positions to the group's largest product and keeps 14 bits below its leading bit,
   truncating the rest (measured; the sums across groups and across MFMAs are fp32).
   So per output element
       |Y_gpu - Y_orc| <= sx*sw*( 7 * 2^-13 * sum_groups max_g|p| + (K/128 + 16) * 2^-24 * sum|p| ) + 2^-22 |Y|
   which the oracle-side quantities bound from above by 7*2^-13*absdot (absdot = scaled sum|p|).
 * bf16 O: <= 2 bf16 ulps, or |delta| <= 2^-13 + (the fp32-Y difference propagated through the
   norm) for values near zero, where cancellation makes an ulp distance meaningless.  The norm
   arithmetic alone (oracle norm of the GPU's own Y) must agree within 1 ulp / 2^-13.
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2605_10886_amd import synth


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    def ordered(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, 0x8000 - u, u)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def check_bf16_out(got_bits, want_bits, max_ulp=2, abs_tol=2.0 ** -13):
    """Pass if every element is within max_ulp bf16 ulps or within abs_tol (scalar or array broadcastable
    to the outputs).  Returns (ok, worst ulp distance among elements judged by ulps, n judged by abs_tol)."""
    d = bf16_ulp_distance(got_bits, want_bits)
    bad = d > max_ulp
    n_abs = int(bad.sum())
    if n_abs:
        g = synth.bits_to_bf16(got_bits).float().numpy()
        w = synth.bits_to_bf16(want_bits).float().numpy()
        tol = np.broadcast_to(np.asarray(abs_tol, dtype=np.float64), d.shape)
        if not (np.abs(g - w)[bad] <= tol[bad]).all():
            return False, int(d.max()), n_abs
    return True, int(d[~bad].max()) if (~bad).any() else 0, n_abs


def propagated_abs_tol(y_orc, dy, norm_kind, eps, gamma=None):
    """Absolute slack of a normalized output caused by the (separately bounded) fp32-Y difference dy:
    to first order |dO| <= rstd * |gamma| * (|dY| + |d mean|) <= 2 * rstd * |gamma| * max_row |dY|,
    on top of 2^-13 for the cancellation of values near zero.  norm_kind: 0 none, 1 LayerNorm, 2 RMSNorm."""
    y = y_orc.astype(np.float64)
    if norm_kind == 1:
        rstd = 1.0 / np.sqrt(y.var(axis=1) + eps)
    elif norm_kind == 2:
        rstd = 1.0 / np.sqrt((y * y).mean(axis=1) + eps)
    else:
        rstd = np.ones(y.shape[0])
    g = np.ones(y.shape[1]) if gamma is None else np.abs(gamma.astype(np.float64))
    return 2.0 ** -13 + 2.0 * rstd[:, None] * g[None, :] * dy.max(axis=1)[:, None]


def propagated_abs_tol_blocknorm(y_orc, dy, block_n, eps, hardswish):
    """Same bound for BlockNorm: rstd is per (row, group of block_n columns); Hard-Swish has slope <= 1.5."""
    y = y_orc.astype(np.float64)
    M, N = y.shape
    g = y.reshape(M, N // block_n, block_n)
    rstd = 1.0 / np.sqrt((g * g).mean(axis=2) + eps)                          # [M, groups]
    dmax = dy.reshape(M, N // block_n, block_n).max(axis=2)                    # [M, groups]
    tol = 2.0 ** -13 + 2.0 * (1.5 if hardswish else 1.0) * rstd * dmax
    return np.repeat(tol, block_n, axis=1)


def gemm_tolerance(absdot: np.ndarray, y_orc: np.ndarray, K: int) -> np.ndarray:
    """Rigorous per-element bound from the oracle's conditioning term (see module docstring)."""
    return (7.0 * 2.0 ** -13 + (K / 128 + 16) * 2.0 ** -24) * absdot + 2.0 ** -22 * np.abs(y_orc.astype(np.float64))


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    a = a.astype(np.float64); b = b.astype(np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def to_np_bits(t: torch.Tensor) -> np.ndarray:
    return synth.bf16_bits(t.cpu())
