"""Thin ctypes binding of libloka.so (the C ABI declared in include/loka.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and the current HIP stream.  There is
no CPU fallback: if the shared library is missing or was not built, every call
raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libloka.so")

LOKA_OK = 0
STATIC_SCRATCH_BYTES = 16 << 20       # LOKA_STATIC_SCRATCH_BYTES of include/loka.h
LOKA_ERR_NULL, LOKA_ERR_SHAPE, LOKA_ERR_ALIGN, LOKA_ERR_UNSUPPORTED = 1, 2, 3, 4
LOKA_ERR_WORKSPACE, LOKA_ERR_HIP, LOKA_ERR_NO_CANDIDATE, LOKA_ERR_TIMEOUT = 5, 6, 7, 8
SCALE_TENSOR, SCALE_ROW, SCALE_COL, SCALE_BLOCK_1x128, SCALE_BLOCK_128x128, SCALE_BLOCK_1x128_POW2, SCALE_BLOCK_128x128_POW2, SCALE_BLOCK_128x1 = range(8)
NORM_NONE, NORM_LAYERNORM, NORM_RMSNORM, NORM_BLOCKNORM = range(4)
NORMS = {"none": NORM_NONE, "layernorm": NORM_LAYERNORM, "rmsnorm": NORM_RMSNORM, "blocknorm": NORM_BLOCKNORM}
ACT_NONE, ACT_HARDSWISH = 0, 1


class GemmDesc(Structure):
    _fields_ = [("M", c_int64), ("N", c_int64), ("K", c_int64), ("batch", c_int64),
                ("strideX", c_int64), ("strideW", c_int64), ("strideO", c_int64),
                ("x_mode", c_int32), ("w_mode", c_int32), ("norm", c_int32), ("eps", c_float),
                ("variant", c_int32), ("block_n", c_int32), ("act", c_int32)]


class ProbeStats(Structure):
    _fields_ = [("rel_fro", c_double), ("max_abs", c_double), ("mere", c_double),
                ("sum_sq_err", c_double), ("sum_sq_ref", c_double)]

    def as_dict(self):
        return {k: float(getattr(self, k)) for k, _ in self._fields_}


class Candidate(Structure):
    _fields_ = [("x_mode", c_int32), ("w_mode", c_int32), ("variant", c_int32), ("feasible", c_int32),
                ("usec", c_float), ("usec_gemm", c_float), ("stats", ProbeStats)]


class Choice(Structure):
    _fields_ = [("x_mode", c_int32), ("w_mode", c_int32), ("variant", c_int32), ("from_cache", c_int32),
                ("usec", c_float), ("usec_bf16", c_float), ("stats", ProbeStats)]


class LokaError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


_lib = None

# every symbol include/loka.h declares: (name, restype, argtypes)
_SIGNATURES = [
    ("loka_status_string", c_char_p, [c_int]),
    ("loka_scale_count", c_int64, [c_int, c_int64, c_int64]),
    ("loka_quantize_workspace", c_size_t, [c_int, c_int64, c_int64, c_int]),
    ("loka_quantize", c_int, [c_void_p, c_int64, c_int64, c_int64, c_int, c_int, c_void_p, c_void_p, c_void_p,
                              c_size_t, c_void_p]),
    ("loka_e4m3_from_f32", c_int, [c_void_p, c_void_p, c_int64, c_void_p]),
    ("loka_machine_ceiling", c_int, [c_int, c_double, c_void_p, c_size_t, POINTER(c_double), c_void_p]),
    ("loka_variant_count", c_int, []),
    ("loka_variant_name", c_char_p, [c_int]),
    ("loka_variant_supports", c_int, [POINTER(GemmDesc), c_int]),
    ("loka_fp8_gemm_norm_workspace", c_size_t, [POINTER(GemmDesc)]),
    ("loka_fp8_gemm_norm", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    ("loka_fp8_linear_norm", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_void_p, c_void_p]),
    ("loka_fp8_linear_norm_xq", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_void_p]),
    ("loka_fp8_gemm_norm_check", c_int, [POINTER(GemmDesc), c_void_p, c_size_t, c_void_p]),
    ("loka_fp8_gemm_norm_static", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p, c_void_p]),
    ("loka_test_set_spin_limit", None, [c_int64]),
    ("loka_fp8_gemm_norm_fp8out_workspace", c_size_t, [POINTER(GemmDesc)]),
    ("loka_fp8_gemm_norm_fp8out", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    ("loka_bf16_gemm_workspace", c_size_t, [POINTER(GemmDesc)]),
    ("loka_bf16_gemm", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    ("loka_probe_error_workspace", c_size_t, [c_int64, c_int64]),
    ("loka_probe_error", c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p,
                                 c_size_t, c_void_p]),
    ("loka_tracker_update_workspace", c_size_t, [c_int64, c_int64]),
    ("loka_tracker_update", c_int, [c_void_p, c_int64, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_size_t,
                                    c_void_p]),
    ("loka_dispatch_select", c_int, [c_int, POINTER(c_double), POINTER(c_double), c_double, c_double, c_double]),
    ("loka_dispatch", c_int, [POINTER(GemmDesc), c_void_p, c_void_p, c_double, c_double, POINTER(Choice),
                              POINTER(Candidate), c_int, POINTER(c_int), c_void_p]),
    ("loka_dispatch_clear", None, []),
    ("loka_default_variant", c_int, [POINTER(GemmDesc)]),
]
EXPORTS = [s[0] for s in _SIGNATURES]


def lib():
    """The loaded library.  Raises if libloka.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2605_10886_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)      # torch is imported above, so the HIP runtime it loaded is shared
        for name, res, args in _SIGNATURES:
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().loka_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != LOKA_OK:
        raise LokaError(status, what)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes: int, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def loka_scale_count(mode: int, rows: int, cols: int) -> int:
    return int(lib().loka_scale_count(mode, rows, cols))


def loka_quantize(x: torch.Tensor, mode: int, transpose_out: bool = False):
    """x bf16 [rows, cols] (device) -> (codes uint8 [rows, cols] or [cols, rows], scales fp32)."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    rows, cols = x.shape
    n = loka_scale_count(mode, rows, cols)
    if n < 0:
        raise LokaError(LOKA_ERR_SHAPE, "loka_scale_count")
    q = torch.empty((cols, rows) if transpose_out else (rows, cols), dtype=torch.uint8, device=x.device)
    s = torch.empty(n, dtype=torch.float32, device=x.device)
    nws = lib().loka_quantize_workspace(mode, rows, cols, int(transpose_out))
    ws = _ws(nws, x.device)
    _check(lib().loka_quantize(_ptr(x), rows, cols, x.stride(0), mode, int(transpose_out), _ptr(q), _ptr(s), _ptr(ws),
                               ws.numel(), _stream()), "loka_quantize")
    return q, s


def loka_e4m3_from_f32(t: torch.Tensor) -> torch.Tensor:
    assert t.dtype == torch.float32 and t.is_contiguous()
    out = torch.empty(t.shape, dtype=torch.uint8, device=t.device)
    _check(lib().loka_e4m3_from_f32(_ptr(t), _ptr(out), t.numel(), _stream()), "loka_e4m3_from_f32")
    return out


def loka_machine_ceiling(kind: int, millis: float, scratch: torch.Tensor) -> float:
    """kind 0 / 1: FP8 / BF16 matrix rate in TFLOP/s; 2: copy rate in GB/s; 3: rate at which the large-layer kernel's operand
    stream reaches the LDS of all CUs, GB/s.  Synchronizes."""
    v = c_double(0.0)
    _check(lib().loka_machine_ceiling(kind, millis, _ptr(scratch), scratch.numel() * scratch.element_size(), byref(v),
                                      _stream()), "loka_machine_ceiling")
    return float(v.value)


def loka_variant_count() -> int:
    return int(lib().loka_variant_count())


def loka_variant_name(v: int):
    r = lib().loka_variant_name(int(v))
    return None if r is None else r.decode()


def variant_id(name: str) -> int:
    for v in range(loka_variant_count()):
        if loka_variant_name(v) == name:
            return v
    raise KeyError(name)


def make_desc(M, N, K, batch=1, x_mode=SCALE_ROW, w_mode=SCALE_COL, norm=NORM_LAYERNORM, eps=1e-5, variant=-1,
              shared_w=False, block_n=0, act=ACT_NONE) -> GemmDesc:
    return GemmDesc(M, N, K, batch, M * K, 0 if shared_w else N * K, M * N, x_mode, w_mode, norm, eps, variant,
                    block_n, act)


def loka_variant_supports(desc: GemmDesc, v: int) -> bool:
    return bool(lib().loka_variant_supports(byref(desc), int(v)))


def loka_default_variant(desc: GemmDesc) -> int:
    return int(lib().loka_default_variant(byref(desc)))


def loka_fp8_gemm_norm(desc: GemmDesc, xq, sx, wq, sw, gamma=None, beta=None, want_y: bool = False, out=None, y=None,
                       workspace=None):
    """Returns (O bf16 [batch*M, N], Y fp32 [batch*M, N] or None)."""
    rows = desc.batch * desc.M
    dev = xq.device
    if out is None:
        out = torch.empty((rows, desc.N), dtype=torch.bfloat16, device=dev)
    if want_y and y is None:
        y = torch.empty((rows, desc.N), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _ws(lib().loka_fp8_gemm_norm_workspace(byref(desc)), dev)
    _check(lib().loka_fp8_gemm_norm(byref(desc), _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), _ptr(gamma), _ptr(beta),
                                    _ptr(out), _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
           "loka_fp8_gemm_norm")
    return out, y


def loka_fp8_linear_norm(desc: GemmDesc, x, wq, sw, gamma=None, beta=None, want_y: bool = False, want_sx: bool = False,
                         out=None):
    """Rowwise quantization of bf16 x fused into the GEMM + norm.  Returns (O bf16, Y fp32 or None, sx or None)."""
    rows = desc.batch * desc.M
    dev = x.device
    if out is None:
        out = torch.empty((rows, desc.N), dtype=torch.bfloat16, device=dev)
    y = torch.empty((rows, desc.N), dtype=torch.float32, device=dev) if want_y else None
    sx = torch.empty(rows, dtype=torch.float32, device=dev) if want_sx else None
    _check(lib().loka_fp8_linear_norm(byref(desc), _ptr(x), _ptr(wq), _ptr(sw), _ptr(gamma), _ptr(beta), _ptr(out), _ptr(y),
                                      _ptr(sx), _stream()), "loka_fp8_linear_norm")
    return out, y, sx


def loka_fp8_linear_norm_xq(desc: GemmDesc, x, wq, sw, gamma=None, beta=None, want_y: bool = False, out=None, xq=None, sx=None):
    """One launch: every workgroup quantizes the rows it consumes (rowwise), then GEMM + norm.  Returns (O bf16, Y fp32 or
    None, xq codes, sx row scales)."""
    rows = desc.batch * desc.M
    dev = x.device
    if out is None:
        out = torch.empty((rows, desc.N), dtype=torch.bfloat16, device=dev)
    if xq is None:
        xq = torch.empty((rows, desc.K), dtype=torch.uint8, device=dev)
    if sx is None:
        sx = torch.empty(rows, dtype=torch.float32, device=dev)
    y = torch.empty((rows, desc.N), dtype=torch.float32, device=dev) if want_y else None
    _check(lib().loka_fp8_linear_norm_xq(byref(desc), _ptr(x), _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), _ptr(gamma), _ptr(beta),
                                         _ptr(out), _ptr(y), _stream()), "loka_fp8_linear_norm_xq")
    return out, y, xq, sx


def loka_fp8_gemm_norm_check(desc: GemmDesc, workspace) -> int:
    """Status of the bounded waits of the last loka_fp8_gemm_norm call on `workspace` (synchronizes): LOKA_OK or
    LOKA_ERR_TIMEOUT."""
    return int(lib().loka_fp8_gemm_norm_check(byref(desc), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                              _stream()))


def loka_fp8_gemm_norm_static(desc: GemmDesc, xq, sx, wq, sw, gamma=None, beta=None, want_y: bool = False, out=None, y=None):
    """loka_fp8_gemm_norm with the library's own scratch (the call allocates nothing; the output tensors here are made
    by the caller of this helper, before the call).  Returns (O bf16, Y fp32 or None)."""
    rows = desc.batch * desc.M
    if out is None:
        out = torch.empty((rows, desc.N), dtype=torch.bfloat16, device=xq.device)
    if want_y and y is None:
        y = torch.empty((rows, desc.N), dtype=torch.float32, device=xq.device)
    _check(lib().loka_fp8_gemm_norm_static(byref(desc), _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), _ptr(gamma), _ptr(beta),
                                           _ptr(out), _ptr(y), _stream()), "loka_fp8_gemm_norm_static")
    return out, y


def loka_test_set_spin_limit(polls: int) -> None:
    lib().loka_test_set_spin_limit(int(polls))


def loka_fp8_gemm_norm_fp8out(desc: GemmDesc, xq, sx, wq, sw, gamma=None, beta=None, want_y: bool = False, oq=None,
                              so=None, y=None, workspace=None):
    """Returns (codes uint8 [batch*M, N], row scales fp32 [batch*M], Y fp32 or None)."""
    rows = desc.batch * desc.M
    dev = xq.device
    if oq is None:
        oq = torch.empty((rows, desc.N), dtype=torch.uint8, device=dev)
    if so is None:
        so = torch.empty(rows, dtype=torch.float32, device=dev)
    if want_y and y is None:
        y = torch.empty((rows, desc.N), dtype=torch.float32, device=dev)
    need = int(lib().loka_fp8_gemm_norm_fp8out_workspace(byref(desc)))
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib().loka_fp8_gemm_norm_fp8out(byref(desc), _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), _ptr(gamma), _ptr(beta),
                                           _ptr(oq), _ptr(so), _ptr(y), _ptr(workspace),
                                           0 if workspace is None else workspace.numel(), _stream()),
           "loka_fp8_gemm_norm_fp8out")
    return oq, so, y


def loka_bf16_gemm(desc: GemmDesc, x, w, yref=None, workspace=None):
    """x bf16 [batch*M, K], w bf16 [batch*K or K, N] -> Yref fp32 [batch*M, N]."""
    dev = x.device
    if yref is None:
        yref = torch.empty((desc.batch * desc.M, desc.N), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _ws(lib().loka_bf16_gemm_workspace(byref(desc)), dev)
    d = GemmDesc(desc.M, desc.N, desc.K, desc.batch, desc.strideX, desc.K * desc.N if desc.strideW else 0,
                 desc.strideO, desc.x_mode, desc.w_mode, desc.norm, desc.eps, desc.variant)
    _check(lib().loka_bf16_gemm(byref(d), _ptr(x), _ptr(w), _ptr(yref), _ptr(workspace), workspace.numel(), _stream()),
           "loka_bf16_gemm")
    return yref


def loka_probe_error(y, yref, stats=None, rowmax=None, workspace=None, sync: bool = True):
    """Returns (stats dict [or the device tensor when sync=False], rowmax fp32 [M])."""
    assert y.dtype == torch.float32 and yref.dtype == torch.float32 and y.shape == yref.shape
    M, N = y.shape
    dev = y.device
    if stats is None:
        stats = torch.empty(5, dtype=torch.float64, device=dev)
    if rowmax is None:
        rowmax = torch.empty(M, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _ws(lib().loka_probe_error_workspace(M, N), dev)
    _check(lib().loka_probe_error(_ptr(y), _ptr(yref), M, N, y.stride(0), _ptr(stats), _ptr(rowmax), _ptr(workspace),
                                  workspace.numel(), _stream()), "loka_probe_error")
    if not sync:
        return stats, rowmax
    v = stats.cpu().tolist()
    return dict(zip(("rel_fro", "max_abs", "mere", "sum_sq_err", "sum_sq_ref"), v)), rowmax


def loka_tracker_update(x: torch.Tensor, n_old: int, mu: torch.Tensor, sigma: torch.Tensor, workspace=None) -> int:
    """Merges the batch x [B, K] bf16 into (n_old, mu [K], sigma [K, K]) in place; returns the new row count."""
    B, K = x.shape
    need = int(lib().loka_tracker_update_workspace(B, K))
    ws = workspace if workspace is not None else _ws(need, x.device)
    _check(lib().loka_tracker_update(_ptr(x), B, K, x.stride(0), int(n_old), _ptr(mu), _ptr(sigma), _ptr(ws), ws.numel(),
                                     _stream()), "loka_tracker_update")
    return int(n_old) + B


def loka_dispatch_select(usec, err, budget: float, min_speedup: float = 0.0, usec_bf16: float = 0.0) -> int:
    n = len(usec)
    a = (c_double * n)(*[float(v) for v in usec])
    b = (c_double * n)(*[float(v) for v in err])
    return int(lib().loka_dispatch_select(n, a, b, budget, min_speedup, usec_bf16))


def loka_dispatch(desc: GemmDesc, x, w, err_budget: float, min_speedup: float = 0.0):
    """Returns (status, choice dict, candidate table list)."""
    choice = Choice()
    cap = 64
    table = (Candidate * cap)()
    n = c_int(0)
    st = lib().loka_dispatch(byref(desc), _ptr(x), _ptr(w), err_budget, min_speedup, byref(choice), table, cap,
                             byref(n), _stream())
    if st not in (LOKA_OK, LOKA_ERR_NO_CANDIDATE):
        raise LokaError(st, "loka_dispatch")
    ch = {"x_mode": choice.x_mode, "w_mode": choice.w_mode, "variant": choice.variant,
          "variant_name": loka_variant_name(choice.variant) if choice.variant >= 0 else None,
          "from_cache": bool(choice.from_cache), "usec": choice.usec, "usec_bf16": choice.usec_bf16,
          "stats": choice.stats.as_dict()}
    rows = [{"x_mode": c.x_mode, "w_mode": c.w_mode, "variant": c.variant, "variant_name": loka_variant_name(c.variant),
             "feasible": bool(c.feasible), "usec": c.usec, "usec_gemm": c.usec_gemm, "stats": c.stats.as_dict()}
            for c in table[:n.value]]
    return st, ch, rows


def loka_dispatch_clear():
    lib().loka_dispatch_clear()
