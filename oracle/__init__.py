"""ctypes front end of the CPU oracle (oracle/loka_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.

All arrays are numpy, C-contiguous.  bf16 tensors travel as uint16 bit patterns,
FP8 codes as uint8.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "loka_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

SCALE_TENSOR, SCALE_ROW, SCALE_COL, SCALE_BLOCK_1x128, SCALE_BLOCK_128x128, SCALE_BLOCK_1x128_POW2, SCALE_BLOCK_128x128_POW2, SCALE_BLOCK_128x1 = range(8)
NORM_NONE, NORM_LAYERNORM, NORM_RMSNORM = range(3)

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (plain -O2, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    c = ctypes
    vp = c.c_void_p
    L.orc_default_threads.restype = c.c_int
    L.orc_bf16_to_f32.restype = c.c_float
    L.orc_bf16_to_f32.argtypes = [c.c_uint16]
    L.orc_f32_to_bf16_rne.restype = c.c_uint16
    L.orc_f32_to_bf16_rne.argtypes = [c.c_float]
    L.orc_e4m3_decode.restype = c.c_double
    L.orc_e4m3_decode.argtypes = [c.c_uint8]
    L.orc_e4m3_encode.restype = c.c_uint8
    L.orc_e4m3_encode.argtypes = [c.c_float]
    L.orc_e4m3_encode_array.restype = None
    L.orc_e4m3_encode_array.argtypes = [vp, vp, c.c_int64]
    L.orc_scale_count.restype = c.c_int64
    L.orc_scale_count.argtypes = [c.c_int, c.c_int64, c.c_int64]
    L.orc_quantize.restype = c.c_int
    L.orc_quantize.argtypes = [vp, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int, vp, vp, c.c_int]
    L.orc_fp8_gemm.restype = c.c_int
    L.orc_fp8_gemm.argtypes = [c.c_int64, c.c_int64, c.c_int64, vp, vp, c.c_int, vp, vp, c.c_int, vp, vp, c.c_int]
    L.orc_tracker_update.restype = c.c_int
    L.orc_tracker_update.argtypes = [vp, c.c_int64, c.c_int64, c.c_int64, vp, vp, vp, c.c_int]
    L.orc_blocknorm.restype = c.c_int
    L.orc_blocknorm.argtypes = [vp, c.c_int64, c.c_int64, c.c_int64, c.c_float, c.c_int, vp, c.c_int]
    L.orc_norm.restype = c.c_int
    L.orc_norm.argtypes = [vp, c.c_int64, c.c_int64, c.c_int, c.c_float, vp, vp, vp, c.c_int]
    L.orc_ref_gemm.restype = c.c_int
    L.orc_ref_gemm.argtypes = [vp, vp, c.c_int64, c.c_int64, c.c_int64, vp, c.c_int]
    L.orc_probe.restype = c.c_int
    L.orc_probe.argtypes = [vp, vp, c.c_int64, c.c_int64, c.c_int64, vp, vp]
    L.orc_dispatch_select.restype = c.c_int
    L.orc_dispatch_select.argtypes = [c.c_int, vp, vp, c.c_double, c.c_double, c.c_double]
    _lib = L
    return L


def default_threads() -> int:
    """Threads the oracle uses when none are given: all host cores, capped by
    OMP_NUM_THREADS when that is set (the GPU machines export their CPU share there)."""
    n = _load().orc_default_threads()
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, n)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, name):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous {dtype}, got {a.dtype}")
    return a


def bf16_to_f32(bits: int) -> float:
    return float(_load().orc_bf16_to_f32(int(bits)))


def f32_to_bf16_rne(f: float) -> int:
    return int(_load().orc_f32_to_bf16_rne(float(np.float32(f))))


def e4m3_decode(code: int) -> float:
    return float(_load().orc_e4m3_decode(int(code)))


def e4m3_encode(t) -> int:
    return int(_load().orc_e4m3_encode(float(np.float32(t))))


def e4m3_encode_array(t: np.ndarray) -> np.ndarray:
    t = np.ascontiguousarray(t, dtype=np.float32)
    out = np.empty(t.shape, dtype=np.uint8)
    _load().orc_e4m3_encode_array(_p(t), _p(out), t.size)
    return out


def scale_count(mode: int, rows: int, cols: int) -> int:
    return int(_load().orc_scale_count(mode, rows, cols))


def quantize(x_bits: np.ndarray, mode: int, transpose_out: bool = False, threads: int | None = None):
    """x_bits: uint16 [rows, cols].  Returns (codes uint8, scales float32)."""
    _chk(x_bits, np.uint16, "x")
    rows, cols = x_bits.shape
    ng = scale_count(mode, rows, cols)
    if ng < 0:
        raise ValueError("scale mode does not divide the shape")
    q = np.empty((cols, rows) if transpose_out else (rows, cols), dtype=np.uint8)
    s = np.empty(ng, dtype=np.float32)
    rc = _load().orc_quantize(_p(x_bits), rows, cols, cols, mode, int(transpose_out), _p(q), _p(s),
                              threads or default_threads())
    if rc:
        raise ValueError("orc_quantize failed")
    return q, s


def fp8_gemm(xq, sx, x_mode, wq, sw, w_mode, want_absdot: bool = False, threads: int | None = None):
    """xq uint8 [M,K], wq uint8 [N,K].  Returns y float32 [M,N] (and absdot float64 [M,N])."""
    _chk(xq, np.uint8, "xq"); _chk(wq, np.uint8, "wq")
    _chk(sx, np.float32, "sx"); _chk(sw, np.float32, "sw")
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    y = np.empty((M, N), dtype=np.float32)
    ad = np.empty((M, N), dtype=np.float64) if want_absdot else None
    rc = _load().orc_fp8_gemm(M, N, K, _p(xq), _p(sx), x_mode, _p(wq), _p(sw), w_mode, _p(y), _p(ad),
                              threads or default_threads())
    if rc:
        raise ValueError("unsupported scale-mode combination")
    return (y, ad) if want_absdot else y


def norm(y, kind: int, eps: float = 1e-5, gamma_bits=None, beta_bits=None, threads: int | None = None):
    """y float32 [M,N] -> bf16 bits uint16 [M,N]."""
    _chk(y, np.float32, "y")
    M, N = y.shape
    out = np.empty((M, N), dtype=np.uint16)
    rc = _load().orc_norm(_p(y), M, N, kind, eps, _p(gamma_bits), _p(beta_bits), _p(out), threads or default_threads())
    if rc:
        raise ValueError("bad norm kind")
    return out


ACT_NONE, ACT_HARDSWISH = 0, 1


def blocknorm(y, block_n: int, eps: float = 1e-5, act: int = ACT_NONE, threads: int | None = None):
    """BlockNorm (unparameterized RMS normalization of consecutive groups of block_n columns) with an optional
    Hard-Swish: y float32 [M,N] -> bf16 bits uint16 [M,N]."""
    _chk(y, np.float32, "y")
    M, N = y.shape
    out = np.empty((M, N), dtype=np.uint16)
    rc = _load().orc_blocknorm(_p(y), M, N, int(block_n), eps, int(act), _p(out), threads or default_threads())
    if rc:
        raise ValueError("block_n must divide N; act in {0, 1}")
    return out


def tracker_update(x_bits, n_old: int, mu, sigma, want_abs: bool = False, threads: int | None = None):
    """Merges the batch x (bf16 bits uint16 [B,K]) into (n_old, mu float32 [K], sigma float32 [K,K]) IN PLACE;
    returns n_new (and the fp64 [K,K] magnitude sum |x_i||x_j| + B|mu_b,i||mu_b,j| when want_abs)."""
    _chk(x_bits, np.uint16, "x"); _chk(mu, np.float32, "mu"); _chk(sigma, np.float32, "sigma")
    Bn, K = x_bits.shape
    assert mu.shape == (K,) and sigma.shape == (K, K)
    ab = np.empty((K, K), dtype=np.float64) if want_abs else None
    rc = _load().orc_tracker_update(_p(x_bits), Bn, K, int(n_old), _p(mu), _p(sigma), _p(ab), threads or default_threads())
    if rc:
        raise ValueError("bad tracker arguments")
    return (n_old + Bn, ab) if want_abs else n_old + Bn


def ref_gemm(x_bits, w_bits, threads: int | None = None):
    """x uint16 [M,K], w uint16 [K,N] (bf16 bits) -> yref float32 [M,N]."""
    _chk(x_bits, np.uint16, "x"); _chk(w_bits, np.uint16, "w")
    M, K = x_bits.shape
    K2, N = w_bits.shape
    assert K == K2
    y = np.empty((M, N), dtype=np.float32)
    _load().orc_ref_gemm(_p(x_bits), _p(w_bits), M, N, K, _p(y), threads or default_threads())
    return y


def probe(y, yref):
    """Returns (stats dict, rowmax float32 [M])."""
    _chk(y, np.float32, "y"); _chk(yref, np.float32, "yref")
    M, N = y.shape
    stats = np.zeros(5, dtype=np.float64)
    rowmax = np.empty(M, dtype=np.float32)
    _load().orc_probe(_p(y), _p(yref), M, N, N, _p(stats), _p(rowmax))
    keys = ("rel_fro", "max_abs", "mere", "sum_sq_err", "sum_sq_ref")
    return dict(zip(keys, (float(v) for v in stats))), rowmax


def dispatch_select(usec, err, budget: float, min_speedup: float = 0.0, usec_baseline: float = 0.0) -> int:
    usec = np.ascontiguousarray(usec, dtype=np.float64)
    err = np.ascontiguousarray(err, dtype=np.float64)
    return int(_load().orc_dispatch_select(len(usec), _p(usec), _p(err), budget, min_speedup, usec_baseline))
