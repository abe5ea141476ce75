"""Host-only checks of the C ABI: the library loads, exports what include/loka.h declares,
and rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_2605_10886_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)           # non-null, 16-byte aligned, never dereferenced on these paths
ODD = ctypes.c_void_p(0x1004)


def _declared():
    text = open(os.path.join(ROOT, "include", "loka.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(loka_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names          # the Python binding covers the same set


def test_status_strings_and_scale_counts():
    assert B.status_string(B.LOKA_OK) == "ok"
    assert "budget" in B.status_string(B.LOKA_ERR_NO_CANDIDATE)
    assert B.loka_scale_count(B.SCALE_TENSOR, 100, 200) == 1
    assert B.loka_scale_count(B.SCALE_ROW, 100, 200) == 100
    assert B.loka_scale_count(B.SCALE_COL, 100, 200) == 200
    assert B.loka_scale_count(B.SCALE_BLOCK_1x128, 100, 256) == 200
    assert B.loka_scale_count(B.SCALE_BLOCK_1x128, 100, 200) == -1
    assert B.loka_scale_count(B.SCALE_BLOCK_128x128, 256, 384) == 6
    assert B.loka_scale_count(B.SCALE_BLOCK_128x128, 100, 384) == -1
    assert B.loka_scale_count(9, 1, 1) == -1 and B.loka_scale_count(B.SCALE_ROW, 0, 5) == -1


def test_variant_table():
    n = B.loka_variant_count()
    assert n >= 4 and B.loka_variant_name(n) is None and B.loka_variant_name(-1) is None
    names = [B.loka_variant_name(v) for v in range(n)]
    assert len(set(names)) == n
    d = B.make_desc(16384, 512, 512, norm=B.NORM_RMSNORM)
    ok = [names[v] for v in range(n) if B.loka_variant_supports(d, v)]
    assert any(s.startswith("row") for s in ok) and not B.loka_variant_supports(d, B.variant_id("row64x256"))
    wide = B.make_desc(32768, 4096, 4096)
    assert all(not names[v].startswith("row") for v in range(n) if B.loka_variant_supports(wide, v))
    assert B.loka_default_variant(d) >= 0 and B.loka_default_variant(wide) >= 0
    bad = B.make_desc(128, 100, 128)                      # N % 16 != 0
    assert B.loka_default_variant(bad) == -1 and not B.loka_variant_supports(bad, 0)


def test_quantize_argument_validation():
    L = B.lib()
    q = L.loka_quantize
    assert q(None, 16, 128, 128, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_NULL
    assert q(FAKE, 16, 128, 128, 8, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_UNSUPPORTED          # no such mode
    assert q(FAKE, 128, 128, 128, B.SCALE_BLOCK_128x1, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_UNSUPPORTED   # needs transpose_out
    assert q(FAKE, 100, 128, 128, B.SCALE_BLOCK_128x1, 1, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_SHAPE         # rows % 128
    assert B.loka_scale_count(B.SCALE_BLOCK_128x1, 256, 48) == 2 * 48
    # a GEMM operand cannot carry that mode (its transposed output is a BLOCK_1x128 operand)
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_BLOCK_128x1)) == B.LOKA_ERR_UNSUPPORTED
    assert q(FAKE, 0, 128, 128, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_SHAPE
    assert q(FAKE, 16, 120, 120, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_SHAPE       # cols % 16
    assert q(FAKE, 16, 128, 64, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_SHAPE        # ld < cols
    assert q(FAKE, 16, 144, 144, B.SCALE_BLOCK_1x128, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_SHAPE
    assert q(FAKE, 16, 128, 132, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_ALIGN       # ld % 8
    assert q(ODD, 16, 128, 128, B.SCALE_ROW, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_ALIGN
    assert q(FAKE, 16, 128, 128, B.SCALE_ROW, 1, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_UNSUPPORTED
    assert q(FAKE, 128, 128, 128, B.SCALE_COL, 1, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_WORKSPACE
    assert q(FAKE, 128, 128, 128, B.SCALE_COL, 1, FAKE, FAKE, FAKE, 8, None) == B.LOKA_ERR_WORKSPACE
    assert L.loka_quantize_workspace(B.SCALE_ROW, 64, 256, 0) == 0
    assert L.loka_quantize_workspace(B.SCALE_COL, 64, 256, 1) == 256 * 8
    assert L.loka_quantize_workspace(B.SCALE_TENSOR, 64, 256, 0) == 8


def _gemm(desc, xq=FAKE, sx=FAKE, wq=FAKE, sw=FAKE, out=FAKE, y=None, ws=None, nws=0):
    return B.lib().loka_fp8_gemm_norm(ctypes.byref(desc), xq, sx, wq, sw, None, None, out, y, ws, nws, None)


def test_gemm_argument_validation():
    good = B.make_desc(256, 128, 128)
    assert _gemm(good, xq=None) == B.LOKA_ERR_NULL
    assert _gemm(good, out=None) == B.LOKA_ERR_NULL
    assert _gemm(B.make_desc(256, 128, 100)) == B.LOKA_ERR_SHAPE            # K % 16
    # the block recipes contract whole 128-wide K blocks
    assert _gemm(B.make_desc(256, 128, 192, x_mode=B.SCALE_BLOCK_1x128, w_mode=B.SCALE_BLOCK_128x128)) == B.LOKA_ERR_SHAPE
    # a K that is a multiple of 16 but not of 128 is a valid shape: some variant takes it, the large-layer and the
    # register-resident kernels do not
    ragged = B.make_desc(2048, 1024, 123200)              # K = 16 * 7700 (Section 2.3's largest shape)
    assert B.loka_default_variant(ragged) >= 0
    assert B.loka_variant_supports(ragged, B.variant_id("row64x1024")) and B.loka_variant_supports(ragged, B.variant_id("twopass128x128"))
    assert not B.loka_variant_supports(ragged, B.variant_id("panel32_256x256")) and not B.loka_variant_supports(ragged, B.variant_id("wreg32"))
    assert _gemm(B.make_desc(256, 120, 128)) == B.LOKA_ERR_SHAPE            # N % 16
    assert _gemm(B.make_desc(0, 128, 128)) == B.LOKA_ERR_SHAPE
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_COL)) == B.LOKA_ERR_UNSUPPORTED
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_BLOCK_1x128)) == B.LOKA_ERR_UNSUPPORTED   # needs 128x128 W
    assert _gemm(B.make_desc(256, 144, 128, x_mode=B.SCALE_BLOCK_1x128, w_mode=B.SCALE_BLOCK_128x128)) == B.LOKA_ERR_SHAPE
    # power-of-two block scales: on both operands or on neither
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_BLOCK_1x128_POW2, w_mode=B.SCALE_BLOCK_128x128)) == B.LOKA_ERR_UNSUPPORTED
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_BLOCK_1x128, w_mode=B.SCALE_BLOCK_128x128_POW2)) == B.LOKA_ERR_UNSUPPORTED
    assert _gemm(B.make_desc(256, 128, 128, x_mode=B.SCALE_ROW, w_mode=B.SCALE_BLOCK_128x128_POW2)) == B.LOKA_ERR_UNSUPPORTED
    assert _gemm(B.make_desc(256, 128, 128, x_mode=7)) == B.LOKA_ERR_UNSUPPORTED
    assert B.loka_scale_count(B.SCALE_BLOCK_1x128_POW2, 256, 512) == 256 * 4
    assert B.loka_scale_count(B.SCALE_BLOCK_128x128_POW2, 256, 512) == 2 * 4
    assert B.loka_scale_count(B.SCALE_BLOCK_128x128_POW2, 200, 512) == -1
    assert _gemm(B.make_desc(256, 128, 128, norm=5)) == B.LOKA_ERR_UNSUPPORTED
    assert _gemm(good, xq=ODD) == B.LOKA_ERR_ALIGN
    narrow = B.make_desc(256, 512, 128, variant=B.variant_id("row64x128"))  # tile narrower than the row
    assert _gemm(narrow) == B.LOKA_ERR_UNSUPPORTED
    two = B.make_desc(256, 2048, 128, variant=B.variant_id("twopass128x128"))
    assert B.lib().loka_fp8_gemm_norm_workspace(ctypes.byref(two)) >= 256 * 2048 * 4
    assert _gemm(two) == B.LOKA_ERR_WORKSPACE
    assert _gemm(two, ws=FAKE, nws=64) == B.LOKA_ERR_WORKSPACE
    grouped = B.make_desc(256, 128, 128, batch=4)
    grouped.strideO = 100
    assert _gemm(grouped) == B.LOKA_ERR_SHAPE


def test_fp8_output_argument_validation():
    L = B.lib()

    def f8(desc, xq=FAKE, oq=FAKE, so=FAKE, ws=None, nws=0):
        return L.loka_fp8_gemm_norm_fp8out(ctypes.byref(desc), xq, FAKE, FAKE, FAKE, None, None, oq, so, None, ws, nws, None)

    panel = B.make_desc(1000, 2048, 512, variant=B.variant_id("panel32_256x256"))
    assert f8(panel, xq=None) == B.LOKA_ERR_NULL
    assert f8(panel, so=None) == B.LOKA_ERR_NULL
    assert f8(panel, oq=ODD) == B.LOKA_ERR_ALIGN
    # records of every row of every 256-row panel, statistics and extremes, two arrival counters per panel, the flag
    need = L.loka_fp8_gemm_norm_fp8out_workspace(ctypes.byref(panel))
    assert need >= 4 * 256 * 8 * 8 * 2 + 2 * 4 * 4 + 256
    assert f8(panel) == B.LOKA_ERR_WORKSPACE
    assert f8(panel, ws=FAKE, nws=need - 1) == B.LOKA_ERR_WORKSPACE
    assert f8(panel, ws=ODD, nws=need) == B.LOKA_ERR_ALIGN
    # kernels that keep the row together need none; a tiled variant has no such epilogue
    assert L.loka_fp8_gemm_norm_fp8out_workspace(ctypes.byref(B.make_desc(1000, 256, 256, variant=B.variant_id("strip32")))) == 0
    assert L.loka_fp8_gemm_norm_fp8out_workspace(ctypes.byref(B.make_desc(1000, 512, 256, variant=B.variant_id("wreg32")))) == 0
    assert f8(B.make_desc(1000, 2048, 512, variant=B.variant_id("twopass128x128"))) == B.LOKA_ERR_UNSUPPORTED
    assert f8(B.make_desc(1000, 2048, 100)) == B.LOKA_ERR_SHAPE


def test_quantize_prologue_argument_validation():
    L = B.lib()

    def xq(desc, x=FAKE, q=FAKE, sx=FAKE, out=FAKE):
        return L.loka_fp8_linear_norm_xq(ctypes.byref(desc), x, q, sx, FAKE, FAKE, None, None, out, None, None)

    skinny = B.make_desc(4096, 512, 512, x_mode=B.SCALE_ROW, w_mode=B.SCALE_COL)
    assert xq(skinny, x=None) == B.LOKA_ERR_NULL
    assert xq(skinny, q=None) == B.LOKA_ERR_NULL
    assert xq(skinny, sx=None) == B.LOKA_ERR_NULL
    assert xq(skinny, q=ODD) == B.LOKA_ERR_ALIGN
    assert xq(B.make_desc(4096, 512, 100, x_mode=B.SCALE_ROW, w_mode=B.SCALE_COL)) == B.LOKA_ERR_SHAPE
    # only with one scale per row of X, only on the streaming kernel and the shapes it covers
    assert xq(B.make_desc(4096, 512, 512, x_mode=B.SCALE_TENSOR, w_mode=B.SCALE_TENSOR)) == B.LOKA_ERR_UNSUPPORTED
    assert xq(B.make_desc(4096, 4096, 4096, x_mode=B.SCALE_ROW, w_mode=B.SCALE_COL)) == B.LOKA_ERR_UNSUPPORTED
    assert xq(B.make_desc(4096, 256, 256, x_mode=B.SCALE_ROW, w_mode=B.SCALE_COL, variant=B.variant_id("strip32"))) == B.LOKA_ERR_UNSUPPORTED
    shared_x = B.make_desc(4096, 256, 256, batch=4, x_mode=B.SCALE_ROW, w_mode=B.SCALE_COL)
    shared_x.strideX = 0
    assert xq(shared_x) == B.LOKA_ERR_UNSUPPORTED


def test_probe_and_bf16_argument_validation():
    L = B.lib()
    assert L.loka_probe_error(None, FAKE, 8, 16, 16, FAKE, None, FAKE, 1 << 20, None) == B.LOKA_ERR_NULL
    assert L.loka_probe_error(FAKE, FAKE, 8, 18, 18, FAKE, None, FAKE, 1 << 20, None) == B.LOKA_ERR_SHAPE
    assert L.loka_probe_error(FAKE, FAKE, 8, 16, 8, FAKE, None, FAKE, 1 << 20, None) == B.LOKA_ERR_SHAPE
    assert L.loka_probe_error(FAKE, FAKE, 8, 16, 16, FAKE, None, None, 0, None) == B.LOKA_ERR_WORKSPACE
    assert L.loka_probe_error(FAKE, ODD, 8, 16, 16, FAKE, None, FAKE, 1 << 20, None) == B.LOKA_ERR_ALIGN
    d = B.make_desc(256, 128, 100)                                          # K % 8 for the BF16 GEMM
    assert L.loka_bf16_gemm(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, 1 << 20, None) == B.LOKA_ERR_SHAPE
    d = B.make_desc(256, 128, 128)
    assert L.loka_bf16_gemm(ctypes.byref(d), FAKE, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_WORKSPACE
    assert L.loka_bf16_gemm_workspace(ctypes.byref(d)) == 128 * 128 * 2
    assert L.loka_e4m3_from_f32(None, FAKE, 4, None) == B.LOKA_ERR_NULL


def test_tracker_argument_validation():
    L = B.lib()
    t = L.loka_tracker_update
    need = L.loka_tracker_update_workspace(1000, 256)
    assert need >= 3 * 128 * 128 * 4                                        # at least one partial per tile pair
    assert L.loka_tracker_update_workspace(1000, 100) == 0                  # K % 8
    assert t(None, 1000, 256, 256, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_NULL
    assert t(FAKE, 1000, 256, 256, 0, None, FAKE, FAKE, need, None) == B.LOKA_ERR_NULL
    assert t(FAKE, 0, 256, 256, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_SHAPE
    assert t(FAKE, 1000, 100, 104, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_SHAPE     # K % 8
    assert t(FAKE, 1000, 256, 128, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_SHAPE     # ld < K
    assert t(FAKE, 1000, 256, 260, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_SHAPE     # ld % 8
    assert t(FAKE, 1000, 256, 256, -1, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_SHAPE
    assert t(ODD, 1000, 256, 256, 0, FAKE, FAKE, FAKE, need, None) == B.LOKA_ERR_ALIGN
    assert t(FAKE, 1000, 256, 256, 0, FAKE, FAKE, None, 0, None) == B.LOKA_ERR_WORKSPACE
    assert t(FAKE, 1000, 256, 256, 0, FAKE, FAKE, FAKE, need - 1, None) == B.LOKA_ERR_WORKSPACE


def test_dispatch_rule_and_validation_on_host():
    assert B.loka_dispatch_select([10, 8, 6, 12], [0.01, 0.03, 0.05, 0.001], 0.04) == 1
    assert B.loka_dispatch_select([10, 8, 6, 12], [0.01, 0.03, 0.05, 0.001], 0.0005) == -1
    assert B.loka_dispatch_select([10, 8], [0.01, 0.01], 0.1, 1.05, 8.2) == -1
    assert B.loka_dispatch_select([10, 8], [0.01, 0.01], 0.1, 1.05, 9.0) == 1
    assert B.loka_dispatch_select([], [], 0.1) == -1
    ch = B.Choice()
    d = B.make_desc(256, 120, 128)
    st = B.lib().loka_dispatch(ctypes.byref(d), FAKE, FAKE, 0.05, 0.0, ctypes.byref(ch), None, 0, None, None)
    assert st == B.LOKA_ERR_SHAPE
    st = B.lib().loka_dispatch(ctypes.byref(d), None, FAKE, 0.05, 0.0, ctypes.byref(ch), None, 0, None, None)
    assert st == B.LOKA_ERR_NULL
    B.loka_dispatch_clear()


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libloka.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_bench_refuses_more_than_one_gpu():
    # the measurement script runs on one GPU: any other count (flag or launcher environment) ends with a message and a
    # non-zero status before anything touches a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
