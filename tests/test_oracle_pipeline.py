"""Pins of the oracle's quantize / GEMM / norm / reference / probe / dispatch functions.

Each function is checked against something other than itself: exact-fraction
re-derivation from the recipe, closed forms, integer-exact cases, brute force
on tiny inputs, and PyTorch / numpy library routines where the operation
reduces to one.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact_model import (bf16_bits_to_fraction, e4m3_code_value, e4m3_nearest_code, e4m3_spacing,
                         round_to_binary32)
from paper_2605_10886_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F448 = Fraction(448)
FLOOR = Fraction(float(np.float32(1e-12)))


# ----------------------------------------------------------------------------- helpers
def exact_quantize(x_bits, mode, orc):
    """Exact-fraction re-derivation of the quantization recipe for a small matrix."""
    rows, cols = x_bits.shape
    xv = [[bf16_bits_to_fraction(int(x_bits[r, c])) for c in range(cols)] for r in range(rows)]

    def gid(r, c):
        return {orc.SCALE_TENSOR: 0, orc.SCALE_ROW: r, orc.SCALE_COL: c,
                orc.SCALE_BLOCK_1x128: r * (cols // 128) + c // 128,
                orc.SCALE_BLOCK_128x128: (r // 128) * (cols // 128) + c // 128,
                orc.SCALE_BLOCK_128x1: c * (rows // 128) + r // 128}[mode]

    ng = orc.scale_count(mode, rows, cols)
    amax = [Fraction(0)] * ng
    for r in range(rows):
        for c in range(cols):
            g = gid(r, c)
            amax[g] = max(amax[g], abs(xv[r][c]))
    amax = [max(a, FLOOR) for a in amax]
    scale = [round_to_binary32(a / F448) for a in amax]
    inv = [round_to_binary32(F448 / a) for a in amax]
    codes = np.zeros((rows, cols), dtype=np.uint8)
    for r in range(rows):
        for c in range(cols):
            t = round_to_binary32(xv[r][c] * inv[gid(r, c)])
            t = max(min(t, F448), -F448)
            neg0 = (int(x_bits[r, c]) >> 15) == 1
            codes[r, c] = e4m3_nearest_code(t, negative_zero=neg0)
    return codes, scale


def f32_bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


DEC = np.array([float(e4m3_code_value(c)) if (c & 0x7F) != 0x7F else np.nan for c in range(256)])


# ----------------------------------------------------------------------------- quantize
def test_golden_2x4_matches_file_and_exact_fractions(orc):
    modes = {"row": orc.SCALE_ROW, "tensor": orc.SCALE_TENSOR, "col": orc.SCALE_COL}
    seen = 0
    for line in open(os.path.join(GOLDEN, "quantize_2x4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, xs, qs, ss = [p.strip() for p in line.split("|")]
        x = np.array([int(v, 16) for v in xs.split()], dtype=np.uint16).reshape(2, 4)
        q_file = np.array([int(v, 16) for v in qs.split()], dtype=np.uint8).reshape(2, 4)
        s_file = np.array([int(v, 16) for v in ss.split()], dtype=np.uint32)
        q, s = orc.quantize(x, modes[name], threads=1)
        assert np.array_equal(q, q_file) and np.array_equal(f32_bits(s), s_file)
        q_exact, s_exact = exact_quantize(x, modes[name], orc)
        assert np.array_equal(q_file, q_exact)
        assert [Fraction(float(v)) for v in s] == s_exact
        seen += 1
    assert seen == 3


@pytest.mark.parametrize("mode_name", ["TENSOR", "ROW", "COL", "BLOCK_1x128", "BLOCK_128x128"])
def test_quantize_every_mode_against_exact_fractions(orc, mode_name):
    mode = getattr(orc, "SCALE_" + mode_name)
    x = synth.student_t4(128, 256, seed=21)
    x[5, :] = 0                                   # an all-zero row
    x[7, 3] = 3.0e4                               # a single large outlier
    xb = synth.bf16_bits(x).copy()
    q, s = orc.quantize(xb, mode, threads=2)
    q_exact, s_exact = exact_quantize(xb, mode, orc)
    assert [Fraction(float(v)) for v in s] == s_exact
    assert np.array_equal(q, q_exact)


def test_quantize_column_blocks_are_the_row_blocks_of_the_transposed_matrix(orc):
    # BLOCK_128x1 (128 consecutive rows of one column share a scale; used for the operands of the weight-gradient GEMM,
    # whose contraction runs over the rows) against (a) exact fractions and (b) its definition: with the output
    # transposed, codes and scales are exactly the 1 x 128 quantization of the transposed matrix, scale for scale
    x = synth.student_t4(256, 48, seed=23)
    x[130:250, 7] = 0                             # an all-zero group (rows 128..255 of column 7 are not all zero: 250..255 stay)
    x[128:256, 9] = 0                             # an all-zero group
    x[3, 11] = 2.5e4
    xb = synth.bf16_bits(x).copy()
    q, s = orc.quantize(xb, orc.SCALE_BLOCK_128x1, threads=2)
    q_exact, s_exact = exact_quantize(xb, orc.SCALE_BLOCK_128x1, orc)
    assert [Fraction(float(v)) for v in s] == s_exact and np.array_equal(q, q_exact)
    qt, st = orc.quantize(xb, orc.SCALE_BLOCK_128x1, transpose_out=True)
    xt = np.ascontiguousarray(xb.T)
    q_ref, s_ref = orc.quantize(xt, orc.SCALE_BLOCK_1x128)
    assert qt.shape == (48, 256) and np.array_equal(qt, q_ref) and np.array_equal(f32_bits(st), f32_bits(s_ref))
    assert np.array_equal(qt, q.T) and np.array_equal(f32_bits(st), f32_bits(s))
    assert s.shape == (2 * 48,) and s[9 * 2 + 1] == np.float32(1e-12) / np.float32(448.0)
    with pytest.raises(ValueError):
        orc.quantize(xb[:200].copy(), orc.SCALE_BLOCK_128x1)


def test_quantize_half_ulp_bound_and_amax_hits_448(orc):
    x = synth.normal(64, 512, seed=2)
    xb = synth.bf16_bits(x)
    q, s = orc.quantize(xb, orc.SCALE_ROW)
    xf = x.float().numpy()
    for r in range(64):
        amax = Fraction(float(np.abs(xf[r]).max()))
        inv = round_to_binary32(F448 / amax)
        c_star = int(np.abs(xf[r]).argmax())
        assert (q[r, c_star] & 0x7F) == 0x7E            # the amax element saturates to +-448
        for c in range(0, 512, 7):
            t = round_to_binary32(Fraction(float(xf[r, c])) * inv)
            t = max(min(t, F448), -F448)
            err = abs(e4m3_code_value(int(q[r, c])) - t)
            assert err <= e4m3_spacing(t) / 2


def test_quantize_power_of_two_scaling_changes_only_the_scale(orc):
    x = synth.normal(16, 256, seed=3)
    xb = synth.bf16_bits(x)
    xb4 = synth.bf16_bits((x.float() * 16.0).to(torch.bfloat16))     # exact in bf16
    for mode in (orc.SCALE_TENSOR, orc.SCALE_ROW, orc.SCALE_COL, orc.SCALE_BLOCK_1x128):
        q1, s1 = orc.quantize(xb, mode)
        q2, s2 = orc.quantize(xb4, mode)
        assert np.array_equal(q1, q2)
        assert np.array_equal(s2, s1 * np.float32(16.0))


def exact_quantize_pow2(x_bits, mode, orc):
    """Power-of-two block modes re-derived in exact fractions: s = the smallest power of two with amax / s <= 448
    (found by stepping, not by logarithms), t = x / s exactly."""
    rows, cols = x_bits.shape
    xv = [[bf16_bits_to_fraction(int(x_bits[r, c])) for c in range(cols)] for r in range(rows)]

    def gid(r, c):
        if mode == orc.SCALE_BLOCK_1x128_POW2:
            return r * (cols // 128) + c // 128
        return (r // 128) * (cols // 128) + c // 128

    ng = orc.scale_count(mode, rows, cols)
    amax = [Fraction(0)] * ng
    for r in range(rows):
        for c in range(cols):
            amax[gid(r, c)] = max(amax[gid(r, c)], abs(xv[r][c]))
    scale = []
    for a in amax:
        a = max(a, FLOOR)
        sc = Fraction(1)
        while a / sc > F448:
            sc *= 2
        while a / (sc / 2) <= F448:
            sc /= 2
        scale.append(sc)
    codes = np.zeros((rows, cols), dtype=np.uint8)
    for r in range(rows):
        for c in range(cols):
            t = xv[r][c] / scale[gid(r, c)]
            assert abs(t) <= F448
            codes[r, c] = e4m3_nearest_code(t, negative_zero=(int(x_bits[r, c]) >> 15) == 1)
    return codes, scale


@pytest.mark.parametrize("mode_name", ["BLOCK_1x128_POW2", "BLOCK_128x128_POW2"])
def test_quantize_power_of_two_modes_against_exact_fractions(orc, mode_name):
    mode = getattr(orc, "SCALE_" + mode_name)
    x = synth.student_t4(128, 256, seed=22)
    x[5, :] = 0                                   # an all-zero row (all-zero 1x128 groups)
    x[7, 3] = 3.0e4                               # a single large outlier
    x[9, 0:128] = 0
    x[9, 17] = 448.0                              # amax / 448 exactly a power of two: the scale is 1, not 2
    x[11, 128:256] = 0
    x[11, 200] = 450.0                            # just above: the scale is 2
    x[13, 0:128] = 0
    x[13, 1] = 448.0 * 2 ** -20                   # exact power of two below one
    xb = synth.bf16_bits(x).copy()
    q, s = orc.quantize(xb, mode, threads=2)
    q_exact, s_exact = exact_quantize_pow2(xb, mode, orc)
    assert [Fraction(float(v)) for v in s] == s_exact
    assert np.array_equal(q, q_exact)
    # every scale is a power of two, and no smaller one would do
    mant, _ = np.frexp(s.astype(np.float64))
    assert np.all(mant == 0.5)
    if mode == orc.SCALE_BLOCK_1x128_POW2:
        assert s.reshape(128, 2)[9, 0] == 1.0 and s.reshape(128, 2)[11, 1] == 2.0 and s.reshape(128, 2)[13, 0] == 2.0 ** -20
        # same group layout as the plain 1x128 mode, scale within [1, 2) of the plain one
        _, s_plain = orc.quantize(xb, orc.SCALE_BLOCK_1x128)
        ratio = s.astype(np.float64) / s_plain.astype(np.float64)
        assert np.all((ratio >= 1.0 - 1e-7) & (ratio < 2.0))


def test_gemm_power_of_two_modes_are_the_block_contraction(orc):
    # the GEMM treats the two power-of-two modes as the block modes (only the scale VALUES differ), rejects a mix
    M, K, N = 8, 256, 128
    x, w = synth.normal(M, K, seed=31), synth.weight(K, N, seed=32)
    xq, sx = orc.quantize(synth.bf16_bits(x), orc.SCALE_BLOCK_1x128_POW2)
    wq, sw = orc.quantize(synth.bf16_bits(w), orc.SCALE_BLOCK_128x128_POW2, transpose_out=True)
    y_p = orc.fp8_gemm(xq, sx, orc.SCALE_BLOCK_1x128_POW2, wq, sw, orc.SCALE_BLOCK_128x128_POW2)
    y_b = orc.fp8_gemm(xq, sx, orc.SCALE_BLOCK_1x128, wq, sw, orc.SCALE_BLOCK_128x128)
    assert np.array_equal(y_p, y_b)
    # brute force in exact fractions on a few outputs
    for (m, n) in [(0, 0), (3, 77), (7, 127)]:
        tot = Fraction(0)
        for kb in range(K // 128):
            part = sum(e4m3_code_value(int(xq[m, k])) * e4m3_code_value(int(wq[n, k])) for k in range(kb * 128, kb * 128 + 128))
            tot += part * Fraction(float(sx[m * (K // 128) + kb])) * Fraction(float(sw[kb * (N // 128) + n // 128]))
        assert abs(Fraction(float(y_p[m, n])) - tot) <= abs(tot) * Fraction(1, 2 ** 23)
    with pytest.raises(ValueError):
        orc.fp8_gemm(xq, sx, orc.SCALE_BLOCK_1x128_POW2, wq, sw, orc.SCALE_BLOCK_128x128)


def test_quantize_zero_matrix(orc):
    xb = np.zeros((4, 128), dtype=np.uint16)
    xb[1, 5] = 0x8000                                               # a negative zero keeps its sign
    q, s = orc.quantize(xb, orc.SCALE_ROW)
    expect = np.zeros((4, 128), dtype=np.uint8)
    expect[1, 5] = 0x80
    assert np.array_equal(q, expect)
    assert np.all(s == np.float32(1e-12) / np.float32(448.0))


def test_quantize_group_structure(orc):
    # each scale group gets its own power-of-two amax, so a wrong group index shows in the scales
    rows, cols = 256, 256
    for mode, shape in ((orc.SCALE_ROW, (rows,)), (orc.SCALE_COL, (cols,)),
                        (orc.SCALE_BLOCK_1x128, (rows, 2)), (orc.SCALE_BLOCK_128x128, (2, 2))):
        x = torch.full((rows, cols), 2.0 ** -8)
        n = int(np.prod(shape))
        expo = (np.arange(n) % 11).reshape(shape)
        if mode == orc.SCALE_ROW:
            x[torch.arange(rows), torch.arange(rows) % cols] = torch.tensor(2.0 ** expo, dtype=torch.float32)
        elif mode == orc.SCALE_COL:
            x[torch.arange(cols) % rows, torch.arange(cols)] = torch.tensor(2.0 ** expo, dtype=torch.float32)
        elif mode == orc.SCALE_BLOCK_1x128:
            for r in range(rows):
                for b in range(2):
                    x[r, b * 128 + (r % 128)] = 2.0 ** int(expo[r, b])
        else:
            for a in range(2):
                for b in range(2):
                    x[a * 128 + 3, b * 128 + 77] = 2.0 ** int(expo[a, b])
        q, s = orc.quantize(synth.bf16_bits(x.to(torch.bfloat16)), mode)
        want = (np.float32(2.0) ** expo.astype(np.float32) / np.float32(448.0)).ravel()
        assert np.array_equal(s, want.astype(np.float32))


def test_quantize_transpose_out(orc):
    xb = synth.bf16_bits(synth.normal(128, 384, seed=8))
    for mode in (orc.SCALE_COL, orc.SCALE_TENSOR, orc.SCALE_BLOCK_128x128):
        q, s = orc.quantize(xb, mode)
        qt, st = orc.quantize(xb, mode, transpose_out=True)
        assert qt.shape == (384, 128) and np.array_equal(qt, q.T) and np.array_equal(s, st)


def test_quantize_rejects_indivisible_block_shapes(orc):
    xb = np.zeros((100, 200), dtype=np.uint16)
    with pytest.raises(ValueError):
        orc.quantize(xb, orc.SCALE_BLOCK_1x128)
    with pytest.raises(ValueError):
        orc.quantize(np.zeros((100, 256), dtype=np.uint16), orc.SCALE_BLOCK_128x128)


# ----------------------------------------------------------------------------- GEMM
def _int_codes(rng, shape, lo=-8, hi=8):
    """Random small integers and their (exact) e4m3 codes."""
    v = rng.integers(lo, hi + 1, size=shape)
    table = {int(e4m3_code_value(c)): c for c in range(0x7F) if e4m3_code_value(c).denominator == 1}
    codes = np.vectorize(lambda i: (table[abs(int(i))] | (0x80 if i < 0 else 0)))(v).astype(np.uint8)
    return v.astype(np.int64), codes


def test_gemm_integer_operands_are_exact(orc):
    rng = np.random.default_rng(1)
    M, N, K = 7, 5, 48
    xi, xq = _int_codes(rng, (M, K))
    wi, wq = _int_codes(rng, (N, K))
    one = np.ones(1, dtype=np.float32)
    y, ad = orc.fp8_gemm(xq, one, orc.SCALE_TENSOR, wq, one, orc.SCALE_TENSOR, want_absdot=True)
    assert np.array_equal(y.astype(np.int64), xi @ wi.T) and y.shape == (M, N)
    assert np.array_equal(ad, (np.abs(xi) @ np.abs(wi).T).astype(np.float64))
    # row and column scales that are powers of two stay exact and land on the right axis
    sx = (2.0 ** rng.integers(-3, 4, size=M)).astype(np.float32)
    sw = (2.0 ** rng.integers(-3, 4, size=N)).astype(np.float32)
    y2 = orc.fp8_gemm(xq, sx, orc.SCALE_ROW, wq, sw, orc.SCALE_COL)
    assert np.array_equal(y2.astype(np.float64), (xi @ wi.T) * sx[:, None].astype(np.float64) * sw[None, :])


def test_gemm_identity_weight_returns_dequantized_input(orc):
    x = synth.normal(9, 32, seed=4)
    xq, sx = orc.quantize(synth.bf16_bits(x), orc.SCALE_ROW)
    wq = np.zeros((32, 32), dtype=np.uint8)
    wq[np.arange(32), np.arange(32)] = 0x38                      # 1.0 on the diagonal
    sw = np.ones(32, dtype=np.float32)
    y = orc.fp8_gemm(xq, sx, orc.SCALE_ROW, wq, sw, orc.SCALE_COL)
    want = (DEC[xq] * sx[:, None].astype(np.float64)).astype(np.float32)
    assert np.array_equal(y, want)


def test_gemm_tiny_against_exact_fractions(orc):
    rng = np.random.default_rng(6)
    M, N, K = 3, 5, 16
    xq = rng.integers(0, 0x7F, size=(M, K)).astype(np.uint8) | (rng.integers(0, 2, size=(M, K)) << 7).astype(np.uint8)
    wq = rng.integers(0, 0x7F, size=(N, K)).astype(np.uint8) | (rng.integers(0, 2, size=(N, K)) << 7).astype(np.uint8)
    sx = rng.uniform(0.001, 0.1, M).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, N).astype(np.float32)
    y = orc.fp8_gemm(xq, sx, orc.SCALE_ROW, wq, sw, orc.SCALE_COL)
    for m in range(M):
        for n in range(N):
            acc = sum(e4m3_code_value(int(xq[m, k])) * e4m3_code_value(int(wq[n, k])) for k in range(K))
            exact = acc * Fraction(float(sx[m])) * Fraction(float(sw[n]))
            want = float(round_to_binary32(exact))
            assert abs(float(y[m, n]) - want) <= abs(want) * 2.0 ** -23, (m, n)


def test_gemm_blockwise_structure_and_equal_scale_reduction(orc):
    rng = np.random.default_rng(12)
    M, N, K = 6, 256, 384
    xi, xq = _int_codes(rng, (M, K), -4, 4)
    wi, wq = _int_codes(rng, (N, K), -4, 4)
    KB, NB = K // 128, N // 128
    # distinct power-of-two scale per block: the result is an exact, hand-computable sum
    sx = (2.0 ** rng.integers(-2, 3, size=(M, KB))).astype(np.float32)
    sw = (2.0 ** rng.integers(-2, 3, size=(KB, NB))).astype(np.float32)
    y = orc.fp8_gemm(xq, sx.ravel(), orc.SCALE_BLOCK_1x128, wq, sw.ravel(), orc.SCALE_BLOCK_128x128)
    want = np.zeros((M, N))
    for kb in range(KB):
        part = xi[:, kb * 128:(kb + 1) * 128] @ wi[:, kb * 128:(kb + 1) * 128].T
        want += part * sx[:, kb][:, None].astype(np.float64) * np.repeat(sw[kb], 128)[None, :]
    assert np.array_equal(y.astype(np.float64), want)
    # all block scales equal: blockwise reduces to per-tensor scaling
    c = np.float32(0.0123)
    yb = orc.fp8_gemm(xq, np.full(M * KB, c, np.float32), orc.SCALE_BLOCK_1x128,
                      wq, np.full(KB * NB, c, np.float32), orc.SCALE_BLOCK_128x128)
    yt = orc.fp8_gemm(xq, np.array([c]), orc.SCALE_TENSOR, wq, np.array([c]), orc.SCALE_TENSOR)
    assert np.allclose(yb, yt, rtol=2.0 ** -22, atol=0)


def test_gemm_blockwise_absdot_is_the_scaled_sum_of_product_magnitudes(orc):
    # absdot scales the element-wise GEMM gate of the block recipes, so it gets pins of its own.
    # (a) integer codes, a distinct power-of-two scale per (row, K block) and (K block, column block): every term
    #     is exact in fp64, so the result must EQUAL sum_kb (|X_kb| |W_kb|^T) sx[m,kb] sw[kb,nb]
    rng = np.random.default_rng(33)
    M, N, K = 5, 256, 256                                        # two K blocks, two column blocks
    xi, xq = _int_codes(rng, (M, K), -6, 6)
    wi, wq = _int_codes(rng, (N, K), -6, 6)
    KB, NB = K // 128, N // 128
    sx = (2.0 ** rng.permutation(np.arange(-5, -5 + M * KB))).reshape(M, KB).astype(np.float32)     # all distinct
    sw = (2.0 ** rng.permutation(np.arange(-2, -2 + KB * NB))).reshape(KB, NB).astype(np.float32)
    y, ad = orc.fp8_gemm(xq, sx.ravel(), orc.SCALE_BLOCK_1x128, wq, sw.ravel(), orc.SCALE_BLOCK_128x128, want_absdot=True)
    want_y = np.zeros((M, N)); want_ad = np.zeros((M, N))
    for kb in range(KB):
        blk = slice(kb * 128, (kb + 1) * 128)
        s = sx[:, kb][:, None].astype(np.float64) * np.repeat(sw[kb], 128)[None, :].astype(np.float64)
        want_y += (xi[:, blk] @ wi[:, blk].T) * s
        want_ad += (np.abs(xi[:, blk]) @ np.abs(wi[:, blk]).T) * s
    assert np.array_equal(y.astype(np.float64), want_y)
    assert np.array_equal(ad, want_ad)
    assert (ad >= np.abs(want_y)).all() and (ad > np.abs(want_y)).any()      # mixed signs: a strict upper bound somewhere
    # swapping the two K blocks' scales of one row changes that row's absdot (the scale sits on the right block)
    sx2 = sx.copy(); sx2[0] = sx2[0, ::-1]
    _, ad2 = orc.fp8_gemm(xq, sx2.ravel(), orc.SCALE_BLOCK_1x128, wq, sw.ravel(), orc.SCALE_BLOCK_128x128, want_absdot=True)
    assert not np.array_equal(ad2[0], ad[0]) and np.array_equal(ad2[1:], ad[1:])
    # (b) arbitrary codes and arbitrary fp32 scales against exact fractions on sampled outputs
    xq = rng.integers(0, 0x7F, size=(M, K)).astype(np.uint8) | (rng.integers(0, 2, size=(M, K)) << 7).astype(np.uint8)
    wq = rng.integers(0, 0x7F, size=(N, K)).astype(np.uint8) | (rng.integers(0, 2, size=(N, K)) << 7).astype(np.uint8)
    sx = rng.uniform(1e-3, 0.2, (M, KB)).astype(np.float32)
    sw = rng.uniform(1e-3, 0.2, (KB, NB)).astype(np.float32)
    y, ad = orc.fp8_gemm(xq, sx.ravel(), orc.SCALE_BLOCK_1x128, wq, sw.ravel(), orc.SCALE_BLOCK_128x128, want_absdot=True)
    for m, n in [(0, 0), (1, 127), (2, 128), (4, 255), (3, 200)]:
        ex_y = ex_a = Fraction(0)
        for kb in range(KB):
            s = Fraction(float(sx[m, kb])) * Fraction(float(sw[kb, n // 128]))
            ps = [e4m3_code_value(int(xq[m, k])) * e4m3_code_value(int(wq[n, k])) for k in range(kb * 128, (kb + 1) * 128)]
            ex_y += sum(ps) * s
            ex_a += sum(abs(p) for p in ps) * s
        assert abs(float(ad[m, n]) - float(ex_a)) <= float(ex_a) * 2.0 ** -48, (m, n)
        assert abs(float(y[m, n]) - float(ex_y)) <= float(ex_a) * 2.0 ** -48 + abs(float(ex_y)) * 2.0 ** -23, (m, n)
    # the non-block recipes' absdot against exact fractions too (row / column scales that are not powers of two)
    sxr = rng.uniform(1e-3, 0.2, M).astype(np.float32); swc = rng.uniform(1e-3, 0.2, N).astype(np.float32)
    _, adr = orc.fp8_gemm(xq, sxr, orc.SCALE_ROW, wq, swc, orc.SCALE_COL, want_absdot=True)
    for m, n in [(0, 3), (4, 250)]:
        ex_a = sum(abs(e4m3_code_value(int(xq[m, k])) * e4m3_code_value(int(wq[n, k]))) for k in range(K))
        ex_a *= Fraction(float(sxr[m])) * Fraction(float(swc[n]))
        assert abs(float(adr[m, n]) - float(ex_a)) <= float(ex_a) * 2.0 ** -48, (m, n)


def test_gemm_rejects_mixed_block_modes(orc):
    z = np.zeros((128, 128), dtype=np.uint8)
    s = np.ones(128, dtype=np.float32)
    with pytest.raises(ValueError):
        orc.fp8_gemm(z, s, orc.SCALE_ROW, z, s, orc.SCALE_BLOCK_128x128)


# ----------------------------------------------------------------------------- norms
def _bf16_ulp_distance(a_bits, b_bits):
    def ordered(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, 0x8000 - u, u)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def test_norm_closed_forms(orc):
    N = 96
    eps = 1e-5
    const = np.full((1, N), 3.25, dtype=np.float32)
    out = orc.norm(const, orc.NORM_LAYERNORM, eps)
    assert np.all(out == 0)                                              # (c - c) / sqrt(eps) = 0
    out = synth.bits_to_bf16(orc.norm(const, orc.NORM_RMSNORM, eps)).float().numpy()
    want = torch.tensor(3.25 / math.sqrt(3.25 ** 2 + eps)).to(torch.bfloat16).float().item()
    assert np.all(out == want)
    alt = np.tile(np.array([2.5, -2.5], dtype=np.float32), N // 2)[None, :]
    out = synth.bits_to_bf16(orc.norm(alt, orc.NORM_LAYERNORM, eps)).float().numpy()
    w = torch.tensor(2.5 / math.sqrt(2.5 ** 2 + eps)).to(torch.bfloat16).float().item()
    assert np.array_equal(out, np.tile(np.array([w, -w], dtype=np.float32), N // 2)[None, :])
    # NORM_NONE is the bf16 rounding of Y
    y = np.random.default_rng(2).standard_normal((3, N)).astype(np.float32)
    got = orc.norm(y, orc.NORM_NONE)
    assert np.array_equal(got, synth.bf16_bits(torch.from_numpy(y).to(torch.bfloat16)))


@pytest.mark.parametrize("affine", [False, True])
def test_norm_against_torch_float64(orc, affine):
    rng = np.random.default_rng(17)
    M, N = 37, 512
    y = (rng.standard_normal((M, N)) * rng.uniform(0.1, 30, (M, 1)) + rng.uniform(-5, 5, (M, 1))).astype(np.float32)
    gamma = beta = None
    gb = bb = None
    if affine:
        g16, b16 = synth.affine(N, seed=5)
        gamma, beta = g16.double(), b16.double()
        gb, bb = synth.bf16_bits(g16), synth.bf16_bits(b16)
    yt = torch.from_numpy(y).double()
    ln = torch.nn.functional.layer_norm(yt, (N,), gamma, beta, eps=1e-5)
    rms = torch.nn.functional.rms_norm(yt, (N,), gamma, eps=1e-5)
    for kind, ref in ((orc.NORM_LAYERNORM, ln), (orc.NORM_RMSNORM, rms)):
        want = synth.bf16_bits(ref.float().to(torch.bfloat16))
        got = orc.norm(y, kind, 1e-5, gb, bb if kind == orc.NORM_LAYERNORM else None)
        d = _bf16_ulp_distance(got, want)
        assert d.max() <= 1 and (d == 0).mean() > 0.999


def test_blocknorm_is_rmsnorm_of_the_reshaped_rows(orc):
    # Section 3.2: BlockNorm = RMSNorm(Y.view(-1, BlockN)).view(B, N), unparameterized
    rng = np.random.default_rng(21)
    M, N = 12, 768
    y = (rng.standard_normal((M, N)) * rng.uniform(0.05, 20, (M, 1))).astype(np.float32)
    y[:, 256:512] *= 37.0                                    # one group with its own magnitude
    for bn in (16, 128, 256, 768):
        got = orc.blocknorm(y, bn, 1e-5)
        # (a) the already pinned RMSNorm of this oracle on the reshaped matrix
        want = orc.norm(np.ascontiguousarray(y.reshape(-1, bn)), orc.NORM_RMSNORM, 1e-5).reshape(M, N)
        assert np.array_equal(got, want)
        # (b) the library routine in fp64
        ref = torch.nn.functional.rms_norm(torch.from_numpy(y).double().view(-1, bn), (bn,), eps=1e-5).view(M, N)
        assert _bf16_ulp_distance(got, synth.bf16_bits(ref.to(torch.bfloat16))).max() <= 1
    # BlockN = N is RMSNorm without gamma
    assert np.array_equal(orc.blocknorm(y, N, 1e-5), orc.norm(y, orc.NORM_RMSNORM, 1e-5))
    # groups do not see each other: changing one group leaves the others' outputs untouched
    y2 = y.copy()
    y2[:, 512:] = rng.standard_normal((M, 256)).astype(np.float32) * 1e3
    a, b = orc.blocknorm(y, 256, 1e-5), orc.blocknorm(y2, 256, 1e-5)
    assert np.array_equal(a[:, :512], b[:, :512]) and not np.array_equal(a[:, 512:], b[:, 512:])
    with pytest.raises(ValueError):
        orc.blocknorm(y, 100)


def test_blocknorm_hardswish_closed_forms_and_library(orc):
    # h-swish(x) = x * ReLU6(x + 3) / 6 (Section 3.2, "Hard Swish"), applied to the normalized value
    bn = 16
    row = np.zeros((4, 2 * bn), dtype=np.float32)
    row[0, :] = 2.0                                          # every group normalizes to 1 -> 1 * 4 / 6
    row[1, 0], row[1, bn] = 5.0, -5.0                        # lone element: +-sqrt(16) = +-4 -> 4 and 0 (both saturated)
    row[2, ::2], row[2, 1::2] = 3.0, -3.0                    # +-1 -> 2/3 and -1/3
    out = synth.bits_to_bf16(orc.blocknorm(row, bn, 0.0, orc.ACT_HARDSWISH)).float().numpy()
    bf = lambda v: torch.tensor(v, dtype=torch.float64).to(torch.bfloat16).float().item()
    assert np.all(out[0] == bf(4.0 / 6.0))
    assert out[1, 0] == 4.0 and out[1, bn] == 0.0 and np.all(out[1, 1:bn] == 0.0)
    assert np.all(out[2, ::2] == bf(2.0 / 3.0)) and np.all(out[2, 1::2] == bf(-1.0 / 3.0))
    out3 = orc.blocknorm(row[3:4], bn, 1e-5, orc.ACT_HARDSWISH)   # an all-zero group (eps > 0): 0 / sqrt(eps) = 0
    assert np.all(out3 == 0)
    # against the library routines in fp64 on random data, every branch of ReLU6 populated
    rng = np.random.default_rng(22)
    y = (rng.standard_normal((64, 512)) * 2.5).astype(np.float32)
    y[:, ::37] *= 6.0
    ref = torch.nn.functional.rms_norm(torch.from_numpy(y).double().view(-1, 256), (256,), eps=1e-5).view(64, 512)
    assert (ref > 3).any() and (ref < -3).any()
    want = torch.nn.functional.hardswish(ref)
    got = orc.blocknorm(y, 256, 1e-5, orc.ACT_HARDSWISH)
    assert _bf16_ulp_distance(got, synth.bf16_bits(want.to(torch.bfloat16))).max() <= 1
    none = orc.blocknorm(y, 256, 1e-5, orc.ACT_NONE)
    assert _bf16_ulp_distance(none, synth.bf16_bits(ref.to(torch.bfloat16))).max() <= 1


# ----------------------------------------------------------------------------- online tracker (Section 3.1)
def _bf16_matrix(rng, rows, cols, loc, scale):
    return (torch.from_numpy(rng.standard_normal((rows, cols)) * scale + loc)).to(torch.bfloat16)


def test_tracker_batches_merge_to_the_covariance_of_all_rows(orc):
    # merging batches one after the other equals the scatter of the concatenation (numpy, fp64); the unbiased
    # covariance is Sigma / (n - 1); batches with different means exercise the delta delta^T term
    rng = np.random.default_rng(41)
    K = 24
    parts = [_bf16_matrix(rng, 40, K, rng.uniform(-3, 3, K), rng.uniform(0.2, 2, K)),
             _bf16_matrix(rng, 7, K, rng.uniform(-3, 3, K) + 5.0, 0.5),
             _bf16_matrix(rng, 129, K, 0.0, 1.0)]
    mu = np.zeros(K, dtype=np.float32)
    sigma = np.zeros((K, K), dtype=np.float32)
    n = 0
    seen = []
    for part in parts:
        n = orc.tracker_update(synth.bf16_bits(part), n, mu, sigma)
        seen.append(part.double().numpy())
        allx = np.concatenate(seen, 0)
        assert n == allx.shape[0]
        np.testing.assert_allclose(mu, allx.mean(0), rtol=2e-7, atol=1e-7)
        c = allx - allx.mean(0)
        np.testing.assert_allclose(sigma, c.T @ c, rtol=5e-7, atol=1e-5)
        np.testing.assert_allclose(sigma / (n - 1), np.cov(allx, rowvar=False), rtol=5e-7, atol=1e-6)
        assert np.array_equal(sigma, sigma.T)
    # one batch or three: same summary up to the fp32 roundings of the stored state
    mu1 = np.zeros(K, dtype=np.float32); s1 = np.zeros((K, K), dtype=np.float32)
    orc.tracker_update(synth.bf16_bits(torch.cat(parts, 0)), 0, mu1, s1)
    np.testing.assert_allclose(s1, sigma, rtol=1e-6, atol=1e-5)
    np.testing.assert_allclose(mu1, mu, rtol=1e-6, atol=1e-7)


def test_tracker_closed_forms(orc):
    K = 8
    # constant columns: zero scatter, mean = the constant; a second batch at another constant: only delta delta^T
    a = torch.full((10, K), 1.5, dtype=torch.bfloat16)
    b = torch.full((30, K), -0.5, dtype=torch.bfloat16)
    mu = np.zeros(K, dtype=np.float32); sg = np.zeros((K, K), dtype=np.float32)
    n = orc.tracker_update(synth.bf16_bits(a), 0, mu, sg)
    assert n == 10 and np.all(mu == 1.5) and np.all(sg == 0)
    n = orc.tracker_update(synth.bf16_bits(b), n, mu, sg)
    assert n == 40 and np.all(mu == 0.0)                              # (10 * 1.5 - 30 * 0.5) / 40
    assert np.all(sg == 10 * 30 / 40 * 4.0)                           # n_old B / n_new * delta^2, delta = -2
    # two points +-1 in one feature: scatter 2 there, 0 elsewhere; abs magnitude is the plain |x||x| sum
    x = torch.zeros((2, K), dtype=torch.bfloat16); x[0, 3], x[1, 3] = 1.0, -1.0
    mu = np.zeros(K, dtype=np.float32); sg = np.zeros((K, K), dtype=np.float32)
    n, ab = orc.tracker_update(synth.bf16_bits(x), 0, mu, sg, want_abs=True)
    want = np.zeros((K, K)); want[3, 3] = 2.0
    assert np.array_equal(sg, want.astype(np.float32)) and np.array_equal(ab, want) and np.all(mu == 0)


def test_tracker_abs_scatter_with_nonzero_column_means(orc):
    # abs_scatter bounds the fp32 accumulation of the GPU's X^T X - B mu mu^T evaluation, so it must be the magnitude
    # of BOTH terms: |X|^T |X| + B |mu_b| |mu_b|^T (numpy, fp64).  Columns with large means of either sign make the
    # second term and the |x| reconstruction matter; a dropped term or a sign slip moves the result by tens of per cent.
    rng = np.random.default_rng(43)
    B_, K = 57, 12
    loc = np.array([9.0, -7.5, 0.0, 3.0, -0.25, 12.0, -12.0, 1.0, 0.0, -4.0, 6.5, 0.5])
    x = _bf16_matrix(rng, B_, K, loc, rng.uniform(0.3, 2.0, K))
    xd = x.double().numpy()
    mub = xd.mean(0)
    mu = np.zeros(K, dtype=np.float32); sg = np.zeros((K, K), dtype=np.float32)
    n, ab = orc.tracker_update(synth.bf16_bits(x), 0, mu, sg, want_abs=True)
    want = np.abs(xd).T @ np.abs(xd) + B_ * np.outer(np.abs(mub), np.abs(mub))
    np.testing.assert_allclose(ab, want, rtol=1e-12, atol=0)
    # each term alone is far from the sum here (so the check above sees either one missing)
    assert (np.abs(xd).T @ np.abs(xd) < 0.75 * want).any() and (B_ * np.outer(np.abs(mub), np.abs(mub)) < 0.75 * want).all()
    # it does bound the two evaluations' magnitudes: |scatter| <= abs_scatter, and it is symmetric
    c = xd - mub
    assert (np.abs(c.T @ c) <= ab * (1 + 1e-12)).all() and np.allclose(ab, ab.T, rtol=1e-13, atol=0)
    # a stored state (second batch) does not enter abs_scatter: it describes the incoming batch only
    x2 = _bf16_matrix(rng, 20, K, -loc, 1.0)
    x2d = x2.double().numpy()
    n2, ab2 = orc.tracker_update(synth.bf16_bits(x2), n, mu, sg, want_abs=True)
    want2 = np.abs(x2d).T @ np.abs(x2d) + 20 * np.outer(np.abs(x2d.mean(0)), np.abs(x2d.mean(0)))
    np.testing.assert_allclose(ab2, want2, rtol=1e-12, atol=0)
    assert n2 == B_ + 20


def test_layernorm_moments_of_fp64_row(orc):
    # after LayerNorm with gamma=1, beta=0 the row has mean 0 and variance var/(var+eps)
    y = (np.random.default_rng(4).standard_normal((8, 1024)) * 0.01).astype(np.float32)   # var ~ 1e-4: eps matters
    out = synth.bits_to_bf16(orc.norm(y, orc.NORM_LAYERNORM, 1e-5)).double().numpy()
    var = y.astype(np.float64).var(axis=1)
    assert np.allclose(out.mean(axis=1), 0, atol=2e-3)
    assert np.allclose(out.var(axis=1), var / (var + 1e-5), rtol=5e-3)


# ----------------------------------------------------------------------------- reference GEMM
def test_ref_gemm_against_torch_float64(orc):
    x = synth.student_t4(33, 192, seed=9)
    w = synth.weight(192, 80, seed=10)
    y = orc.ref_gemm(synth.bf16_bits(x), synth.bf16_bits(w))
    want = (x.double() @ w.double())
    assert y.shape == (33, 80)
    # fp64 sums differ from the library's only in their last bits; after rounding to fp32 they agree
    # except for rare boundary cases of one fp32 ulp
    diff = np.abs(y.astype(np.float64) - want.numpy())
    assert np.all(diff <= np.abs(want.numpy()) * 2.0 ** -23 + 1e-12)
    assert (y == want.float().numpy()).mean() > 0.999


def test_ref_gemm_integer_exact_and_orientation(orc):
    rng = np.random.default_rng(3)
    xi = rng.integers(-9, 10, size=(4, 24))
    wi = rng.integers(-9, 10, size=(24, 6))
    xb = synth.bf16_bits(torch.from_numpy(xi).to(torch.bfloat16))
    wb = synth.bf16_bits(torch.from_numpy(wi).to(torch.bfloat16))
    y = orc.ref_gemm(xb, wb)
    assert np.array_equal(y.astype(np.int64), xi @ wi)


# ----------------------------------------------------------------------------- probe
def test_probe_zero_and_single_perturbation(orc):
    rng = np.random.default_rng(0)
    M, N = 12, 40
    ref = rng.standard_normal((M, N)).astype(np.float32)
    st, rm = orc.probe(ref.copy(), ref)
    assert st["rel_fro"] == 0 and st["max_abs"] == 0 and st["mere"] == 0 and np.all(rm == 0)
    y = ref.copy()
    y[5, 7] = ref[5, 7] + np.float32(0.5)
    d = np.float32(y[5, 7]) - ref[5, 7]
    st, rm = orc.probe(y, ref)
    ssr = float((ref.astype(np.float64) ** 2).sum())
    assert math.isclose(st["rel_fro"], abs(float(d)) / math.sqrt(ssr), rel_tol=1e-14)
    assert st["max_abs"] == abs(float(d)) and rm[5] == abs(d) and np.count_nonzero(rm) == 1
    assert math.isclose(st["mere"], abs(float(d)) / abs(float(ref[5, 7])) / (M * N), rel_tol=1e-14)
    assert math.isclose(st["sum_sq_ref"], ssr, rel_tol=1e-14)
    # a zero reference element uses the floored denominator instead of dividing by zero
    ref2 = ref.copy(); ref2[0, 0] = 0
    y2 = ref2.copy(); y2[0, 0] = np.float32(1e-3)
    st2, _ = orc.probe(y2, ref2)
    assert math.isclose(st2["mere"], float(np.float32(1e-3)) / 1e-30 / (M * N), rel_tol=1e-12)


def test_probe_against_numpy(orc):
    rng = np.random.default_rng(8)
    ref = rng.standard_normal((64, 96)).astype(np.float32)
    y = (ref + 0.03 * rng.standard_normal((64, 96))).astype(np.float32)
    st, rm = orc.probe(y, ref)
    d = (y - ref).astype(np.float64)
    assert math.isclose(st["rel_fro"], np.linalg.norm(d) / np.linalg.norm(ref.astype(np.float64)), rel_tol=1e-12)
    assert np.array_equal(rm, np.abs(y - ref).max(axis=1))
    assert st["max_abs"] == float(np.abs(y - ref).max())
    assert math.isclose(st["mere"], float(np.mean(np.abs(d) / np.abs(ref.astype(np.float64)))), rel_tol=1e-12)


def test_probe_magnitudes_of_the_fp8_path(orc):
    # e4m3 has 3 mantissa bits: rel-Frobenius error of the quantized GEMM is a few 1e-2 whatever K is,
    # and a bf16-rounded output alone is ~1.7e-3.  MERE (heavy-tailed) is a few 1e-1 for FP8, the order
    # of magnitude of the paper's Table "Geometric mean of MERE" (0.47-0.56 FP8, 0.03-0.04 BF16).
    x = synth.normal(256, 256, seed=31)
    w = synth.weight(256, 192, seed=32)
    xb, wb = synth.bf16_bits(x), synth.bf16_bits(w)
    yref = orc.ref_gemm(xb, wb)
    xq, sx = orc.quantize(xb, orc.SCALE_ROW)
    wq, sw = orc.quantize(wb, orc.SCALE_COL, transpose_out=True)
    y = orc.fp8_gemm(xq, sx, orc.SCALE_ROW, wq, sw, orc.SCALE_COL)
    st, _ = orc.probe(y, yref)
    assert 0.02 < st["rel_fro"] < 0.05
    assert 0.03 < st["mere"] < 3.0
    y16 = torch.from_numpy(yref).to(torch.bfloat16).float().numpy()
    st16, _ = orc.probe(y16, yref)
    assert 1.0e-3 < st16["rel_fro"] < 2.5e-3
    assert st16["mere"] < st["mere"] / 5


# ----------------------------------------------------------------------------- dispatch rule
def test_dispatch_rule_on_fake_tables(orc):
    usec = [10.0, 8.0, 6.0, 12.0]
    err = [0.01, 0.03, 0.05, 0.001]
    assert orc.dispatch_select(usec, err, budget=0.04) == 1
    assert orc.dispatch_select(usec, err, budget=0.06) == 2
    assert orc.dispatch_select(usec, err, budget=0.02) == 0
    assert orc.dispatch_select(usec, err, budget=0.0005) == -1                 # empty feasible set
    # the speedup filter removes candidates that are not enough faster than the baseline
    assert orc.dispatch_select(usec, err, budget=0.06, min_speedup=1.05, usec_baseline=6.2) == -1
    assert orc.dispatch_select(usec, err, budget=0.06, min_speedup=1.05, usec_baseline=9.0) == 2
    assert orc.dispatch_select(usec, err, budget=0.04, min_speedup=1.05, usec_baseline=9.0) == 1
    assert orc.dispatch_select([5.0, 5.0], [0.01, 0.01], budget=0.1) == 0      # ties: lowest index
