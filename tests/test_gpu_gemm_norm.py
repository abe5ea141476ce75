"""GPU parity of loka_fp8_gemm_norm (and loka_bf16_gemm) against the CPU oracle.

The GPU consumes the codes and scales its own loka_quantize produced; those are
checked bit-exact against the oracle first, so both sides contract the same operands.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth
from parity_util import (check_bf16_out, check_fp32_y, propagated_abs_tol, propagated_abs_tol_blocknorm, rel_fro,
                         to_np_bits)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RECIPES = {"tensor": (B.SCALE_TENSOR, B.SCALE_TENSOR), "row": (B.SCALE_ROW, B.SCALE_COL),
           "block": (B.SCALE_BLOCK_1x128, B.SCALE_BLOCK_128x128),
           "block_pow2": (B.SCALE_BLOCK_1x128_POW2, B.SCALE_BLOCK_128x128_POW2)}


# Caps on the rel-Frobenius distance of fp32 Y from the oracle at full size: at most twice what was measured on MI355X
# (C2 2.2e-5, C3 1.4e-5, C5 row / block / tensor 5.7e-5 / 5.0e-5 / 7.1e-5: the matrix pipe's truncation on that data;
# heavier tails and outlier channels widen the spread of product magnitudes inside a group of 8).  The sharper,
# data-dependent gates are in parity_util.check_fp32_y.
FRO_CAP = {"C2": 4.4e-5, "C3": 2.8e-5, "C5 row": 1.14e-4, "C5 block": 1.0e-4, "C5 block_pow2": 1.5e-4, "C5 tensor": 1.42e-4}


def _variants_for(desc):
    return [v for v in range(B.loka_variant_count()) if B.loka_variant_supports(desc, v)]


def _run_case(orc, x, w, recipe, norm, variant, gamma=None, beta=None, rows=None, tag="", fro_cap=None):
    """One problem, full GPU run; oracle on `rows` (all when None).  Returns measured error figures."""
    M, K = x.shape
    N = w.shape[1]
    xm, wm = RECIPES[recipe]
    xd, wd = x.to(DEV), w.to(DEV)
    xq, sx = B.loka_quantize(xd, xm)
    wq, sw = B.loka_quantize(wd, wm, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, xm, wm, B.NORMS[norm], 1e-5, variant)
    gd = None if gamma is None else gamma.to(DEV)
    bd = None if beta is None else beta.to(DEV)
    out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gd, bd, want_y=True)
    out2, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gd, bd, want_y=False)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)), f"{tag}: O differs with/without the Y store"

    # oracle on the same operands (its own quantization, checked equal to the GPU's)
    sel = np.arange(M) if rows is None else np.asarray(rows)
    xb = synth.bf16_bits(x)
    if xm == B.SCALE_TENSOR:
        xq_o, sx_o = orc.quantize(xb, xm)
        xq_o = xq_o[sel]
    else:
        xq_o, sx_o = orc.quantize(xb[sel].copy(), xm)
    wq_o, sw_o = orc.quantize(synth.bf16_bits(w), wm, transpose_out=True)
    idx = torch.from_numpy(sel).to(DEV)
    assert np.array_equal(xq[idx].cpu().numpy(), xq_o), f"{tag}: X codes"
    assert np.array_equal(wq.cpu().numpy(), wq_o), f"{tag}: W codes"
    sx_g = sx.cpu().numpy()
    if xm == B.SCALE_ROW:
        sx_g = sx_g[sel]
    elif xm in (B.SCALE_BLOCK_1x128, B.SCALE_BLOCK_1x128_POW2):
        sx_g = sx_g.reshape(M, K // 128)[sel].ravel()
    assert np.array_equal(sx_g, sx_o) and np.array_equal(sw.cpu().numpy(), sw_o), f"{tag}: scales"

    y_o, absdot = orc.fp8_gemm(np.ascontiguousarray(xq_o), sx_o, xm, wq_o, sw_o, wm, want_absdot=True)
    y_g = y[idx].cpu().numpy()
    exact = variant >= 0 and B.loka_variant_name(variant).startswith("exact")
    fig = check_fp32_y(y_g, y_o, absdot, xq_o, sx_o, xm, wq_o, sw_o, wm, K, tag, None if exact else fro_cap, exact=exact)
    err = fig.pop("err")

    gb = None if gamma is None else synth.bf16_bits(gamma)
    bb = None if beta is None else synth.bf16_bits(beta)
    o_o = orc.norm(y_o, B.NORMS[norm], 1e-5, gb, bb)
    o_g = to_np_bits(out[idx])
    gam = None if gamma is None else gamma.float().numpy()
    ok, worst_ulp, n_abs = check_bf16_out(o_g, o_o, abs_tol=propagated_abs_tol(y_o, err, B.NORMS[norm], 1e-5, gam))
    assert ok, f"{tag}: bf16 O beyond 2 ulps (worst {worst_ulp})"
    # isolate the norm arithmetic: the oracle's norm of the GPU's own Y must match within 1 ulp
    o_iso = orc.norm(np.ascontiguousarray(y_g), B.NORMS[norm], 1e-5, gb, bb)
    ok1, w1, _ = check_bf16_out(o_g, o_iso, max_ulp=1)
    assert ok1, f"{tag}: norm arithmetic alone is off by {w1} ulps"
    return dict(fig, o_worst_ulp=worst_ulp, o_abs_clause=n_abs)


# ----------------------------------------------------------------------------- small shapes, every variant
@pytest.mark.parametrize("recipe", ["tensor", "row", "block", "block_pow2"])
@pytest.mark.parametrize("norm", ["layernorm", "rmsnorm", "none"])
def test_c1_every_variant(orc, recipe, norm):
    w = synth.WORKLOADS["C1"]
    x, wt = synth.activations(w), synth.weights(w)
    xm, wm = RECIPES[recipe]
    desc = B.make_desc(w.M, w.N, w.K, 1, xm, wm, B.NORMS[norm])
    vs = _variants_for(desc)
    assert vs
    for v in vs:
        _run_case(orc, x, wt, recipe, norm, v, tag=f"C1 {recipe} {norm} {B.loka_variant_name(v)}")


@pytest.mark.parametrize("shape", [(200, 128, 48), (77, 256, 240), (333, 384, 512), (130, 128, 1008), (64, 512, 2048),
                                   (100, 512, 256), (90, 1024, 112), (300, 1024, 240),
                                   # rows wider than a tile with 5 and 10 (ragged) tiles per row: the persistent grid is
                                   # then not a multiple of 8 and a panel's workgroups sit on several XCDs
                                   (700, 256, 1280), (520, 128, 2320)])
def test_ragged_tiles_every_variant(orc, shape):
    # M not a multiple of any tile height, N not a multiple of the tile width (but of 16), several K steps
    M, K, N = shape
    x = synth.student_t4(M, K, seed=M)
    wt = synth.weight(K, N, seed=N)
    gamma, beta = synth.affine(N, seed=3)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM)
    for v in _variants_for(desc):
        _run_case(orc, x, wt, "row", "layernorm", v, gamma, beta, tag=f"{shape} LN {B.loka_variant_name(v)}")
        _run_case(orc, x, wt, "row", "rmsnorm", v, gamma, None, tag=f"{shape} RMS {B.loka_variant_name(v)}")


@pytest.mark.parametrize("shape", [(200, 144, 128), (333, 400, 512), (130, 1008, 256), (90, 112, 1024), (77, 16, 48),
                                   (300, 2000, 1280), (64, 4080, 2320)])
def test_ragged_k_every_variant(orc, shape):
    # K a multiple of 16 but not of the kernels' 128-byte K step: the last step's tail is masked in both operands.
    # Codes past the end of a row must not leak in: the operands are cut out of larger matrices whose neighbouring
    # elements are NaN codes after quantization would be impossible, so X and W are laid out with a following row that
    # starts with large values instead (a leak changes the result far beyond the tolerance).
    M, K, N = shape
    x = synth.student_t4(M, K, seed=M + K)
    wt = synth.weight(K, N, seed=N + K)
    x[:, :16] *= 50.0                                  # the bytes that follow a row's end in memory are the next row's start
    gamma, beta = synth.affine(N, seed=4)
    for recipe in ("row", "tensor"):
        desc = B.make_desc(M, N, K, 1, *RECIPES[recipe], B.NORM_LAYERNORM)
        vs = _variants_for(desc)
        names = {B.loka_variant_name(v) for v in vs}
        assert vs and not (names & {"panel32_256x256", "wreg32", "strip32"})
        assert B.loka_default_variant(desc) in vs
        for v in vs:
            _run_case(orc, x, wt, recipe, "layernorm", v, gamma, beta, tag=f"{shape} {recipe} LN {B.loka_variant_name(v)}")
            _run_case(orc, x, wt, recipe, "none", v, tag=f"{shape} {recipe} none {B.loka_variant_name(v)}")
    # the block recipes need whole 128-wide K blocks
    if K % 128:
        with pytest.raises(B.LokaError):
            B.loka_fp8_gemm_norm(B.make_desc(M, 128, K, 1, *RECIPES["block"], B.NORM_NONE),
                                 torch.zeros(M, K, dtype=torch.uint8, device=DEV), torch.ones(M, device=DEV),
                                 torch.zeros(128, K, dtype=torch.uint8, device=DEV), torch.ones(128, device=DEV))


def test_ragged_k_largest_shape_of_the_throughput_study(orc):
    # Section 2.3, "Throughput Analysis": the study's shapes run up to (2048, 123200) @ (123200, 1024); K = 16 * 7700.
    # Full size on the GPU, the oracle on sampled rows; the library's own choice of kernel and the dispatcher's table.
    M, K, N = 2048, 123200, 1024
    x = synth.normal(M, K, seed=21)
    wt = synth.weight(K, N, seed=22)
    rows = _sample_rows(M, 8)[::4]
    # (ranges of several hundred K steps: the two-stage form of the split-K schedule is the static choice)
    assert B.loka_variant_name(B.loka_default_variant(B.make_desc(M, N, K, 1, norm=B.NORM_LAYERNORM))) == "splitk128x128s2"
    r = _run_case(orc, x, wt, "row", "layernorm", -1, rows=rows, tag="2048x123200x1024")
    print("2048x123200x1024", r)
    st, ch, table = B.loka_dispatch(B.make_desc(M, N, K, 1, norm=B.NORM_LAYERNORM), x.to(DEV), wt.to(DEV), 5e-2)
    assert st == B.LOKA_OK and ch["variant"] >= 0
    print("dispatch 2048x123200x1024:", ch["variant_name"], [(t["variant_name"], round(t["usec_gemm"])) for t in table])
    B.loka_dispatch_clear()


@pytest.mark.parametrize("case", [(256, 16384, 1024, "row", "none"), (256, 16384, 1024, "block", "none"),
                                  (512, 8192, 512, "tensor", "layernorm"), (300, 4096, 2320, "row", "rmsnorm"),
                                  (128, 32768, 256, "block_pow2", "layernorm"),
                                  (300, 4096, 640, "block", "layernorm")])      # block scales with a ragged last row tile
@pytest.mark.parametrize("form", ["splitk128x128", "splitk128x128s2"])
def test_split_k_few_tiles_long_k(orc, case, form):
    # few output tiles and a long K (the shape of a weight-gradient GEMM, or of a wide layer at small batch): several
    # workgroups per tile contract a K range each, a second kernel adds the partial sums in a fixed order and normalizes.
    # Two forms of the main kernel: a ring of four LDS stages (the choice for ranges of up to 128 K steps, as here) and
    # the two-stage loop (long ranges)
    M, K, N, recipe, norm = case
    x = synth.student_t4(M, K, seed=5 * M)
    wt = synth.weight(K, N, seed=5 * N)
    gamma, beta = synth.affine(N, seed=9) if norm != "none" else (None, None)
    v = B.variant_id(form)
    desc = B.make_desc(M, N, K, 1, *RECIPES[recipe], B.NORMS[norm], 1e-5, v)
    assert B.loka_variant_supports(desc, v)
    assert B.loka_variant_name(B.loka_default_variant(B.make_desc(M, N, K, 1, *RECIPES[recipe], B.NORMS[norm]))) == "splitk128x128"
    r = _run_case(orc, x, wt, recipe, norm, v, gamma, beta if norm == "layernorm" else None, tag=f"split-K {case}")
    print("split-K", case, r)
    # repeatable bits: the partial sums are added in a fixed order
    xq, sx = B.loka_quantize(x.to(DEV), RECIPES[recipe][0])
    wq, sw = B.loka_quantize(wt.to(DEV), RECIPES[recipe][1], transpose_out=True)
    a, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    for _ in range(3):
        b, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # not offered where K would not be split
    assert not B.loka_variant_supports(B.make_desc(32768, 4096, 4096, 1, variant=v), v)
    assert not B.loka_variant_supports(B.make_desc(256, 128, 128, 1, variant=v), v)


@pytest.mark.parametrize("recipe", ["block", "block_pow2"])
def test_blockwise_ragged(orc, recipe):
    M, K, N = 150, 384, 640
    x, _ = synth.normal_outlier4(M, K, seed=8)
    x[3, 128:256] *= 2.0 ** -30                  # block scales 30 binades apart within one row
    x[5, 0:128] = 0
    wt = synth.weight(K, N, seed=9)
    wt[128:256, 0:128] *= 2.0 ** 12              # and within one column block of W
    desc = B.make_desc(M, N, K, 1, *RECIPES[recipe], B.NORM_LAYERNORM)
    for v in _variants_for(desc):
        _run_case(orc, x, wt, recipe, "layernorm", v, tag=f"{recipe} {B.loka_variant_name(v)}")
        _run_case(orc, x, wt, recipe, "none", v, tag=f"{recipe} no norm {B.loka_variant_name(v)}")


def test_layernorm_rows_with_large_mean(orc):
    # rows whose mean is far larger than their spread: the fused statistics must not cancel
    M, K, N = 64, 128, 256
    x = (synth.normal(M, K, seed=1).float() * 0.05 + 3.0).to(torch.bfloat16)
    wt = (synth.weight(K, N, seed=2).float().abs() + 0.05).to(torch.bfloat16)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM)
    for v in _variants_for(desc):
        _run_case(orc, x, wt, "row", "layernorm", v, tag=f"large-mean {B.loka_variant_name(v)}")


def test_scale_invariance_of_fused_norm():
    # multiplying a row of X by a power of two changes sx only: codes and normalized output stay identical
    # (RMSNorm / LayerNorm are invariant to input scaling up to eps)
    M, K, N = 64, 256, 256
    x = synth.normal(M, K, seed=4)
    x2 = (x.float() * 8.0).to(torch.bfloat16)
    wt = synth.weight(K, N, seed=5).to(DEV)
    wq, sw = B.loka_quantize(wt, B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, eps=0.0)
    q1, s1 = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    q2, s2 = B.loka_quantize(x2.to(DEV), B.SCALE_ROW)
    assert torch.equal(q1, q2) and torch.equal(s2, s1 * 8.0)
    o1, _ = B.loka_fp8_gemm_norm(desc, q1, s1, wq, sw)
    o2, _ = B.loka_fp8_gemm_norm(desc, q2, s2, wq, sw)
    d = (o1.float() - o2.float()).abs().max().item()
    assert d <= 2.0 ** -7                                     # at most 1 bf16 ulp at |o| ~ 1


# ----------------------------------------------------------------------------- benchmark configurations, full size
def _sample_rows(M, n=192):
    rng = np.random.default_rng(M)
    return np.unique(np.concatenate([np.arange(40), rng.integers(0, M, n), np.arange(M - 40, M)]))


def test_c2_full_size_both_recipes(orc):
    w = synth.WORKLOADS["C2"]
    x, wt = synth.activations(w), synth.weights(w)
    for recipe in ("row", "tensor"):
        r = _run_case(orc, x, wt, recipe, w.norm, -1, rows=_sample_rows(w.M, 512), tag=f"C2 {recipe}", fro_cap=FRO_CAP["C2"])
        print("C2", recipe, r)


def test_c3_skinny_pair_chained(orc):
    # layer a's LayerNorm output (bf16, from the GPU) is layer b's input, as in the configuration
    wa, wb = synth.WORKLOADS["C3a"], synth.WORKLOADS["C3b"]
    x, w1, w2 = synth.activations(wa), synth.weights(wa), synth.weights(wb)
    rows = _sample_rows(wa.M, 160)
    r = _run_case(orc, x, w1, "row", "layernorm", -1, rows=rows, tag="C3a", fro_cap=FRO_CAP["C3"])
    print("C3a", r)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    wq, sw = B.loka_quantize(w1.to(DEV), B.SCALE_COL, transpose_out=True)
    da = B.make_desc(wa.M, wa.N, wa.K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM)
    h, _ = B.loka_fp8_gemm_norm(da, xq, sx, wq, sw)
    r = _run_case(orc, h.cpu(), w2, "row", "layernorm", -1, rows=rows, tag="C3b", fro_cap=FRO_CAP["C3"])
    print("C3b", r)


@pytest.mark.parametrize("name", ["C2", "C3a", "C3b", "C4"])
def test_exact_product_variants_full_size(orc, name):
    # the accuracy-first candidates (e4m3 widened to bf16 in registers, BF16 matrix instruction): fp32 Y within the
    # stated 1e-5 of the ORACLE, per element (relative to sum |terms|) and in rel-Frobenius, at the configurations' full
    # sizes; bf16 O within 2 ulps
    w = synth.WORKLOADS[name]
    x = synth.activations(w) if name != "C3b" else synth.normal(w.M, w.K, seed=w.seed)
    wt = synth.weights(w)
    desc = B.make_desc(w.M, w.N, w.K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORMS[w.norm])
    vs = [v for v in _variants_for(desc) if B.loka_variant_name(v).startswith("exact")]
    assert vs
    for v in vs:
        for recipe in ("row", "tensor") if name == "C2" else ("row",):
            r = _run_case(orc, x, wt, recipe, w.norm, v, rows=_sample_rows(w.M, 96), tag=f"{name} {recipe} {B.loka_variant_name(v)}")
            print(name, recipe, B.loka_variant_name(v), r)
            assert r["y_rel_fro"] <= 1e-5


@pytest.mark.parametrize("variant", [None, "strip32", "wreg32"])
def test_c4_grouped_launch(orc, variant):
    w = synth.WORKLOADS["C4"]
    G = w.batch
    xs = torch.cat([synth.activations(w, g) for g in range(G)], 0)          # [G*M, K]
    ws = torch.cat([synth.weights(w, g) for g in range(G)], 0)              # [G*K, N]
    xd, wd = xs.to(DEV), ws.to(DEV)
    xq, sx = B.loka_quantize(xd, B.SCALE_ROW)                               # row-local: all groups at once
    wq = torch.empty(G * w.N, w.K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * w.N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s = B.loka_quantize(wd[g * w.K:(g + 1) * w.K], B.SCALE_COL, transpose_out=True)
        wq[g * w.N:(g + 1) * w.N] = q
        sw[g * w.N:(g + 1) * w.N] = s
    desc = B.make_desc(w.M, w.N, w.K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM,
                       variant=-1 if variant is None else B.variant_id(variant))
    out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, want_y=True)
    torch.cuda.synchronize()
    for g in (0, 1, 31, 63):
        rows = _sample_rows(w.M, 64)
        xb = synth.bf16_bits(xs[g * w.M:(g + 1) * w.M])[rows].copy()
        xq_o, sx_o = orc.quantize(xb, B.SCALE_ROW)
        wq_o, sw_o = orc.quantize(synth.bf16_bits(ws[g * w.K:(g + 1) * w.K]), B.SCALE_COL, transpose_out=True)
        y_o, absdot = orc.fp8_gemm(xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, want_absdot=True)
        idx = torch.from_numpy(rows + g * w.M).to(DEV)
        assert np.array_equal(xq[idx].cpu().numpy(), xq_o)
        y_g = y[idx].cpu().numpy()
        err = check_fp32_y(y_g, y_o, absdot, xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, w.K, f"group {g}", 2.8e-5)["err"]
        o_o = orc.norm(y_o, B.NORM_RMSNORM)
        ok, worst, _ = check_bf16_out(to_np_bits(out[idx]), o_o,
                                      abs_tol=propagated_abs_tol(y_o, err, B.NORM_RMSNORM, 1e-5))
        assert ok, f"group {g}: worst {worst} ulps"
    # a single weight shared by all groups (strideW = 0) must equal group 0's weight applied to every group
    # (same kernel variant for both launches: the order of the row-statistics sums differs between variants)
    v = B.loka_default_variant(desc) if variant is None else B.variant_id(variant)
    desc0 = B.make_desc(w.M, w.N, w.K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, variant=v, shared_w=True)
    out_s, _ = B.loka_fp8_gemm_norm(desc0, xq, sx, wq[:w.N], sw[:w.N])
    d1 = B.make_desc(w.M, w.N, w.K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, variant=v)
    out_1, _ = B.loka_fp8_gemm_norm(d1, xq[5 * w.M:6 * w.M], sx[5 * w.M:6 * w.M], wq[:w.N], sw[:w.N])
    assert torch.equal(out_s[5 * w.M:6 * w.M].view(torch.int16), out_1.view(torch.int16))


@pytest.mark.parametrize("variant", ["wreg32", "strip32"])
def test_streaming_variant_crosses_problem_boundaries(orc, variant):
    # 300 small problems with their own weights: with one row block per problem and fewer workgroups than
    # blocks, some workgroups walk from one problem into the next and must reload W and re-request X
    G, M, K, N = 300, 64, 256, 256
    v = B.variant_id(variant)
    xs = torch.cat([synth.normal(M, K, seed=1000 + g) for g in range(G)], 0)
    ws = torch.cat([synth.weight(K, N, seed=5000 + g) for g in range(G)], 0)
    gamma, beta = synth.affine(N, seed=11)
    xd, wd = xs.to(DEV), ws.to(DEV)
    xq, sx = B.loka_quantize(xd, B.SCALE_ROW)
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s = B.loka_quantize(wd[g * K:(g + 1) * K], B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, variant=v)
    assert B.loka_variant_supports(desc, v)
    out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True)
    out2, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma.to(DEV), beta.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    gb, bb = synth.bf16_bits(gamma), synth.bf16_bits(beta)
    for g in (0, 1, 127, 128, 255, 256, 257, 299):
        xq_o, sx_o = orc.quantize(synth.bf16_bits(xs[g * M:(g + 1) * M]), B.SCALE_ROW)
        wq_o, sw_o = orc.quantize(synth.bf16_bits(ws[g * K:(g + 1) * K]), B.SCALE_COL, transpose_out=True)
        assert np.array_equal(xq[g * M:(g + 1) * M].cpu().numpy(), xq_o)
        y_o, absdot = orc.fp8_gemm(xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, want_absdot=True)
        y_g = y[g * M:(g + 1) * M].cpu().numpy()
        err = check_fp32_y(y_g, y_o, absdot, xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, K, f"problem {g}")["err"]
        o_o = orc.norm(y_o, B.NORM_LAYERNORM, 1e-5, gb, bb)
        ok, worst, _ = check_bf16_out(to_np_bits(out[g * M:(g + 1) * M]), o_o,
                                      abs_tol=propagated_abs_tol(y_o, err, B.NORM_LAYERNORM, 1e-5, gamma.float().numpy()))
        assert ok, f"problem {g}: worst {worst} ulps"


@pytest.mark.parametrize("variant,N", [("wreg32", 512), ("wreg32", 1024), ("strip32", 256)])
def test_streaming_variant_without_norm_many_blocks(orc, variant, N):
    # several row blocks per workgroup and no normalization: nothing but the kernel's own barriers separates one
    # block's output staging from the next block's.  O must be the bf16 rounding of Y everywhere (bit-exact),
    # with and without the fp32 output, and Y must match the oracle on sampled rows.
    M, K = 40000 + 17, 256
    v = B.variant_id(variant)
    x, w = synth.normal(M, K, seed=77), synth.weight(K, N, seed=78)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    wq, sw = B.loka_quantize(w.to(DEV), B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_NONE, variant=v)
    assert B.loka_variant_supports(desc, v)
    out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, want_y=True)
    torch.cuda.synchronize()
    for _ in range(3):
        out2, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
        torch.cuda.synchronize()
        assert torch.equal(out2.view(torch.int16), y.to(torch.bfloat16).view(torch.int16))
    assert torch.equal(out.view(torch.int16), y.to(torch.bfloat16).view(torch.int16))
    rows = np.unique(np.concatenate([np.arange(0, 70), np.arange(M - 70, M), np.arange(0, M, 997)]))
    xq_o, sx_o = orc.quantize(synth.bf16_bits(x[rows]), B.SCALE_ROW)
    wq_o, sw_o = orc.quantize(synth.bf16_bits(w), B.SCALE_COL, transpose_out=True)
    assert np.array_equal(xq[torch.from_numpy(rows).to(DEV)].cpu().numpy(), xq_o)
    y_o, absdot = orc.fp8_gemm(xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, want_absdot=True)
    check_fp32_y(y[torch.from_numpy(rows).to(DEV)].cpu().numpy(), y_o, absdot, xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o,
                 B.SCALE_COL, K, f"{variant} N={N}")


# ----------------------------------------------------------------------------- BlockNorm + Hard-Swish
def _run_blocknorm_case(orc, x, w, recipe, act, variant, rows=None, tag=""):
    M, K = x.shape
    N = w.shape[1]
    xm, wm = RECIPES[recipe]
    xq, sx = B.loka_quantize(x.to(DEV), xm)
    wq, sw = B.loka_quantize(w.to(DEV), wm, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, xm, wm, B.NORM_BLOCKNORM, 1e-5, variant, block_n=256, act=act)
    out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, want_y=True)
    out2, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)), f"{tag}: O differs with/without the Y store"
    sel = np.arange(M) if rows is None else np.asarray(rows)
    idx = torch.from_numpy(sel).to(DEV)
    xb = synth.bf16_bits(x)
    if xm == B.SCALE_TENSOR:
        xq_o, sx_o = orc.quantize(xb, xm)
        xq_o = xq_o[sel]
    else:
        xq_o, sx_o = orc.quantize(xb[sel].copy(), xm)
    wq_o, sw_o = orc.quantize(synth.bf16_bits(w), wm, transpose_out=True)
    assert np.array_equal(xq[idx].cpu().numpy(), xq_o) and np.array_equal(wq.cpu().numpy(), wq_o), f"{tag}: codes"
    y_o, absdot = orc.fp8_gemm(np.ascontiguousarray(xq_o), sx_o, xm, wq_o, sw_o, wm, want_absdot=True)
    y_g = y[idx].cpu().numpy()
    err = check_fp32_y(y_g, y_o, absdot, xq_o, sx_o, xm, wq_o, sw_o, wm, K, tag)["err"]
    o_o = orc.blocknorm(y_o, 256, 1e-5, act)
    o_g = to_np_bits(out[idx])
    ok, worst, n_abs = check_bf16_out(o_g, o_o, abs_tol=propagated_abs_tol_blocknorm(y_o, err, 256, 1e-5, act == B.ACT_HARDSWISH))
    assert ok, f"{tag}: bf16 O beyond 2 ulps (worst {worst})"
    o_iso = orc.blocknorm(np.ascontiguousarray(y_g), 256, 1e-5, act)       # norm + activation arithmetic alone
    ok1, w1, _ = check_bf16_out(o_g, o_iso, max_ulp=1)
    assert ok1, f"{tag}: norm arithmetic alone is off by {w1} ulps"
    return worst


@pytest.mark.parametrize("act", [B.ACT_NONE, B.ACT_HARDSWISH])
@pytest.mark.parametrize("shape", [(300, 256, 256), (200, 128, 512), (130, 256, 1024), (77, 384, 768), (513, 1024, 256)])
def test_blocknorm_every_variant(orc, shape, act):
    M, K, N = shape
    x = synth.student_t4(M, K, seed=M + 1)
    wt = synth.weight(K, N, seed=N + 1)
    for recipe in ("row", "tensor", "block"):
        xm, wm = RECIPES[recipe]
        desc = B.make_desc(M, N, K, 1, xm, wm, B.NORM_BLOCKNORM, block_n=256, act=act)
        vs = _variants_for(desc)
        assert vs and all(B.loka_variant_name(v) in ("wreg32", "panel32_256x256") for v in vs)
        assert B.loka_default_variant(desc) in vs
        for v in vs:
            _run_blocknorm_case(orc, x, wt, recipe, act, v, tag=f"{shape} {recipe} act{act} {B.loka_variant_name(v)}")


def test_blocknorm_rejects_what_is_not_built():
    d = B.make_desc(256, 512, 256, 1, norm=B.NORM_BLOCKNORM, block_n=128)
    assert not any(B.loka_variant_supports(d, v) for v in range(B.loka_variant_count()))
    d = B.make_desc(256, 384, 256, 1, norm=B.NORM_BLOCKNORM, block_n=256)       # N not a multiple of the group
    assert not any(B.loka_variant_supports(d, v) for v in range(B.loka_variant_count()))
    d = B.make_desc(256, 512, 256, 1, norm=B.NORM_RMSNORM, act=B.ACT_HARDSWISH)  # activation only with BlockNorm
    assert not any(B.loka_variant_supports(d, v) for v in range(B.loka_variant_count()))


def test_blocknorm_c5_full_size(orc):
    w = synth.WORKLOADS["C5"]
    x, wt = synth.activations(w), synth.weights(w)
    r = _run_blocknorm_case(orc, x, wt, "row", B.ACT_HARDSWISH, -1, rows=_sample_rows(w.M, 96), tag="C5 blocknorm")
    print("C5 blocknorm + hardswish: worst ulp", r)


# ----------------------------------------------------------------------------- FP8 output for the next layer
@pytest.mark.parametrize("variant", ["wreg32", "strip32"])
@pytest.mark.parametrize("case", [(300, 256, 256, "layernorm"), (200, 128, 512, "rmsnorm"), (130, 256, 1024, "layernorm"),
                                  (513, 1024, 256, "none"), (96, 512, 512, "blocknorm"), (1000, 128, 112, "rmsnorm"),
                                  (20000, 256, 240, "layernorm"), (9000, 512, 128, "layernorm")])
def test_fp8_output_equals_quantize_of_the_bf16_output(orc, case, variant):
    # the fused epilogue must write exactly what loka_quantize(O_bf16, ROW) writes (codes and scales bit for
    # bit); O_bf16 itself is checked against the oracle by the tests above, and the oracle's quantize of the
    # same bf16 tensor is compared as well
    M, K, N, norm = case
    x = synth.student_t4(M, K, seed=7 * M)
    wt = synth.weight(K, N, seed=7 * N)
    gamma, beta = synth.affine(N, seed=5)
    v = B.variant_id(variant)
    kw = dict(block_n=256, act=B.ACT_HARDSWISH) if norm == "blocknorm" else {}
    if not B.loka_variant_supports(B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, v, **kw), v):
        pytest.skip(f"{variant} does not cover this case")
    for xm, wm in ((B.SCALE_ROW, B.SCALE_COL), (B.SCALE_TENSOR, B.SCALE_TENSOR)):
        xq, sx = B.loka_quantize(x.to(DEV), xm)
        wq, sw = B.loka_quantize(wt.to(DEV), wm, transpose_out=True)
        desc = B.make_desc(M, N, K, 1, xm, wm, B.NORMS[norm], 1e-5, v, **kw)
        out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True)
        oq, so, y2 = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True)
        torch.cuda.synchronize()
        assert torch.equal(y, y2)
        q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
        assert torch.equal(oq, q_ref), f"{case} codes differ from loka_quantize of the bf16 output"
        assert torch.equal(so.view(torch.int32), s_ref.view(torch.int32)), f"{case} scales differ"
        q_o, s_o = orc.quantize(to_np_bits(out), B.SCALE_ROW)
        assert np.array_equal(oq.cpu().numpy(), q_o) and np.array_equal(so.cpu().numpy(), s_o)


@pytest.mark.parametrize("variant", ["wreg32", "strip32"])
def test_fp8_output_grouped_launch(orc, variant):
    # several problems with their own weights in one launch, ragged row count: codes and scales of every problem equal
    # loka_quantize of that launch's bf16 output
    G, M, K, N = 5, 650, 256, 256
    v = B.variant_id(variant)
    x = torch.cat([synth.normal(M, K, 900 + g) for g in range(G)], 0).to(DEV)
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s_ = B.loka_quantize(synth.weight(K, N, 950 + g).to(DEV), B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s_
    xq, sx = B.loka_quantize(x, B.SCALE_ROW)
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, 1e-5, v)
    out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw)
    torch.cuda.synchronize()
    q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
    assert torch.equal(oq, q_ref) and torch.equal(so.view(torch.int32), s_ref.view(torch.int32))
    q_o, s_o = orc.quantize(to_np_bits(out), orc.SCALE_ROW)                # the oracle's quantization of that output
    assert np.array_equal(oq.cpu().numpy(), q_o) and np.array_equal(so.cpu().numpy().view(np.uint32), s_o.view(np.uint32))


def test_fp8_output_chains_the_skinny_pair(orc):
    # C3 at reduced M: layer a writes codes + row scales, layer b consumes them directly
    wa, wb = synth.WORKLOADS["C3a"], synth.WORKLOADS["C3b"]
    M = 4096
    x = synth.activations(wa, rows=M)
    w1, w2 = synth.weights(wa), synth.weights(wb)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    w1q, s1 = B.loka_quantize(w1.to(DEV), B.SCALE_COL, transpose_out=True)
    w2q, s2 = B.loka_quantize(w2.to(DEV), B.SCALE_COL, transpose_out=True)
    v = B.variant_id("wreg32")
    da = B.make_desc(M, wa.N, wa.K, 1, norm=B.NORM_LAYERNORM, variant=v)
    db = B.make_desc(M, wb.N, wb.K, 1, norm=B.NORM_LAYERNORM, variant=v)
    hq, hs, _ = B.loka_fp8_gemm_norm_fp8out(da, xq, sx, w1q, s1)
    out_fused, _ = B.loka_fp8_gemm_norm(db, hq, hs, w2q, s2)
    h, _ = B.loka_fp8_gemm_norm(da, xq, sx, w1q, s1)                       # the unfused chain: bf16 through HBM
    hq2, hs2 = B.loka_quantize(h, B.SCALE_ROW)
    out_ref, _ = B.loka_fp8_gemm_norm(db, hq2, hs2, w2q, s2)
    torch.cuda.synchronize()
    assert torch.equal(hq, hq2) and torch.equal(hs, hs2)
    assert torch.equal(out_fused.view(torch.int16), out_ref.view(torch.int16))
    hq_o, hs_o = orc.quantize(to_np_bits(h), orc.SCALE_ROW)               # the hand-over is the oracle's quantization of h
    assert np.array_equal(hq.cpu().numpy(), hq_o) and np.array_equal(hs.cpu().numpy().view(np.uint32), hs_o.view(np.uint32))


# the large-layer kernel: a row spans several workgroups; the row extremes travel with the row statistics
PANEL_FP8_CASES = [
    (700, 512, 1024, "layernorm"),        # 4 tiles per row, ragged last row panel
    (1300, 256, 4096, "rmsnorm"),         # 16 tiles per row: both halves of the tile fold, several panels per workgroup slot
    (520, 384, 2320, "layernorm"),        # ragged last column tile (2320 = 9 * 256 + 16)
    (300, 1024, 256, "layernorm"),        # one tile per row: no exchange, finalized in the tile
    (260, 128, 176, "rmsnorm"),           # one ragged tile, a single K step
    (66000, 128, 512, "layernorm"),       # more row panels than the persistent grid has slots
]


@pytest.mark.parametrize("affine", [False, True])
@pytest.mark.parametrize("case", PANEL_FP8_CASES)
def test_fp8_output_of_the_panel_kernel(orc, case, affine):
    # codes and row scales bit for bit what loka_quantize(O_bf16, ROW) writes from the same kernel's bf16 output
    # (itself checked against the oracle above), and what the oracle's quantize makes of that tensor.  Without gamma /
    # beta the row extremes travel with the statistics (one exchange); with them the row amax of the affine result
    # crosses the workgroups in a second exchange.
    M, K, N, norm = case
    x = synth.student_t4(M, K, seed=11 * M)
    wt = synth.weight(K, N, seed=11 * N)
    gamma, beta = (t.to(DEV) for t in synth.affine(N, seed=6)) if affine else (None, None)
    v = B.variant_id("panel32_256x256")
    for xm, wm in ((B.SCALE_ROW, B.SCALE_COL), (B.SCALE_TENSOR, B.SCALE_TENSOR)):
        xq, sx = B.loka_quantize(x.to(DEV), xm)
        wq, sw = B.loka_quantize(wt.to(DEV), wm, transpose_out=True)
        desc = B.make_desc(M, N, K, 1, xm, wm, B.NORMS[norm], 1e-5, v)
        out, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma, beta, want_y=True)
        need = B.lib().loka_fp8_gemm_norm_fp8out_workspace(desc)
        assert (need > 0) == (N > 256)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
        oq, so, y2 = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, gamma, beta, want_y=True, workspace=ws)
        torch.cuda.synchronize()
        assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
        assert torch.equal(y, y2)
        q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
        assert torch.equal(so.view(torch.int32), s_ref.view(torch.int32)), f"{case} scales differ"
        assert torch.equal(oq, q_ref), f"{case} codes differ from loka_quantize of the bf16 output"
        if M <= 2000:
            q_o, s_o = orc.quantize(to_np_bits(out), B.SCALE_ROW)
            assert np.array_equal(oq.cpu().numpy(), q_o) and np.array_equal(so.cpu().numpy(), s_o)


@pytest.mark.parametrize("affine", [False, True])
def test_fp8_output_of_the_panel_kernel_c5_full_size(orc, affine):
    # the launch bench.py's C5pair times: 128 row panels x 16 tiles on the persistent grid, 8 rounds per workgroup
    # (with gamma / beta: two exchanges per tile)
    w = synth.WORKLOADS["C5"]
    x, wt = synth.activations(w), synth.weights(w)
    gamma, beta = (t.to(DEV) for t in synth.affine(w.N, seed=12)) if affine else (None, None)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt.to(DEV), B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(w.M, w.N, w.K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORMS[w.norm], w.eps, B.variant_id("panel32_256x256"))
    out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma, beta)
    ws = torch.empty(B.lib().loka_fp8_gemm_norm_fp8out_workspace(desc), dtype=torch.uint8, device=DEV)
    oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, gamma, beta, workspace=ws)
    torch.cuda.synchronize()
    assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
    q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
    assert torch.equal(so.view(torch.int32), s_ref.view(torch.int32))
    assert torch.equal(oq, q_ref)
    rows = _sample_rows(w.M, 64)                      # and the oracle's quantize on sampled rows of that bf16 output
    idx = torch.as_tensor(rows, device=DEV)
    q_o, s_o = orc.quantize(to_np_bits(out[idx].contiguous()), B.SCALE_ROW)
    assert np.array_equal(oq[idx].cpu().numpy(), q_o) and np.array_equal(so[idx].cpu().numpy(), s_o)


@pytest.mark.parametrize("variant,shape", [("wreg32", (200, 256, 512)), ("strip32", (200, 256, 256)),
                                           ("panel32_256x256", (300, 256, 768))])
@pytest.mark.parametrize("norm", ["layernorm", "rmsnorm"])
def test_fp8_output_degenerate_rows(orc, variant, shape, norm):
    # rows of zeros (amax 0: the scale falls back to the clamp, codes are all zero), a row with one huge element, a row
    # of one repeated value (LayerNorm output exactly zero), negative-only rows (the row minimum decides the scale)
    M, K, N = shape
    x = synth.normal(M, K, seed=77)
    x[3] = 0
    x[M - 1] = 0
    x[10] = 0
    x[10, 5] = 3.0e4
    x[20] = 0.5
    x[30] = -x[30].abs()
    wt = synth.weight(K, N, seed=78)
    wt[:, : N // 2] = wt[:, : N // 2].abs()                      # half of the outputs of row 30 certainly negative
    v = B.variant_id(variant)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt.to(DEV), B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, v)
    out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw)
    torch.cuda.synchronize()
    q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
    assert torch.equal(so.view(torch.int32), s_ref.view(torch.int32))
    assert torch.equal(oq, q_ref)
    assert int(oq[3].max()) == 0 and int(oq[M - 1].max()) == 0   # zero rows: zero codes
    assert float(so[3]) == float(s_ref[3]) > 0.0
    # against the oracle: its quantization of this bf16 output gives the same codes and scales bit for bit, and the bf16
    # output itself is the oracle's (GEMM on the oracle's own codes, norm) within 2 ulps, degenerate rows included
    q_o, s_o = orc.quantize(to_np_bits(out), orc.SCALE_ROW)
    assert np.array_equal(oq.cpu().numpy(), q_o) and np.array_equal(so.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
    xq_o, sx_o = orc.quantize(synth.bf16_bits(x), orc.SCALE_ROW)
    wq_o, sw_o = orc.quantize(synth.bf16_bits(wt), orc.SCALE_COL, transpose_out=True)
    assert np.array_equal(xq.cpu().numpy(), xq_o)
    y_o, absdot = orc.fp8_gemm(xq_o, sx_o, orc.SCALE_ROW, wq_o, sw_o, orc.SCALE_COL, want_absdot=True)
    o_o = orc.norm(y_o, B.NORMS[norm], 1e-5)
    # (Y is not returned by this call: bound its difference by the operands' truncation bound)
    dy = 7 * 2.0 ** -13 * absdot
    ok, worst, _ = check_bf16_out(to_np_bits(out), o_o, abs_tol=propagated_abs_tol(y_o, dy, B.NORMS[norm], 1e-5))
    assert ok, f"bf16 O beyond 2 ulps of the oracle (worst {worst})"
    assert np.all(o_o[3] == 0) and np.all(to_np_bits(out)[3] & 0x7FFF == 0)        # zero row: (0 - 0) / sqrt(eps)
    assert s_o[3] == np.float32(1e-12) / np.float32(448.0)                          # the amax floor sets its scale
    # row 10 (a single huge input): its FP8 row scale is set by the largest normalized value, on both sides
    q_oo, s_oo = orc.quantize(o_o, orc.SCALE_ROW)
    assert np.allclose(so.cpu().numpy(), s_oo, rtol=2.0 ** -6, atol=0)


@pytest.mark.parametrize("act", [B.ACT_NONE, B.ACT_HARDSWISH])
@pytest.mark.parametrize("shape", [(700, 512, 1024), (1300, 256, 4096), (300, 1024, 256), (520, 384, 2304)])
def test_fp8_output_of_the_panel_kernel_under_blocknorm(orc, shape, act):
    # BlockNorm's statistics stay inside a tile (loka_fp8_gemm_norm needs no workspace), the row amax of the FP8 output
    # crosses the tiles: the exchange after the normalization, on its own
    M, K, N = shape
    x, wt = synth.student_t4(M, K, seed=13 * M), synth.weight(K, N, seed=13 * N)
    v = B.variant_id("panel32_256x256")
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt.to(DEV), B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_BLOCKNORM, 1e-5, v, block_n=256, act=act)
    assert B.lib().loka_fp8_gemm_norm_workspace(desc) == 0
    need = B.lib().loka_fp8_gemm_norm_fp8out_workspace(desc)
    assert (need > 0) == (N > 256)
    out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    for _ in range(2):                                   # the same workspace twice
        oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, workspace=ws)
        torch.cuda.synchronize()
        assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
        q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
        assert torch.equal(so.view(torch.int32), s_ref.view(torch.int32))
        assert torch.equal(oq, q_ref)
    q_o, s_o = orc.quantize(to_np_bits(out), B.SCALE_ROW)
    assert np.array_equal(oq.cpu().numpy(), q_o) and np.array_equal(so.cpu().numpy(), s_o)


def test_fp8_output_of_the_panel_kernel_grouped_and_repeated():
    # several problems in one launch; the same workspace serves consecutive launches (counters cleared by the launch)
    G, M, K, N = 3, 530, 256, 768
    v = B.variant_id("panel32_256x256")
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s_ = B.loka_quantize(synth.weight(K, N, 960 + g).to(DEV), B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s_
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5, v)
    ws = torch.empty(B.lib().loka_fp8_gemm_norm_fp8out_workspace(desc), dtype=torch.uint8, device=DEV)
    for rep in range(3):
        x = torch.cat([synth.normal(M, K, 970 + 10 * rep + g) for g in range(G)], 0).to(DEV)
        xq, sx = B.loka_quantize(x, B.SCALE_ROW)
        gamma, beta = (t.to(DEV) for t in synth.affine(N, seed=rep)) if rep % 2 else (None, None)   # both forms, same workspace
        out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma, beta)
        oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, gamma, beta, workspace=ws)
        torch.cuda.synchronize()
        assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
        q_ref, s_ref = B.loka_quantize(out, B.SCALE_ROW)
        assert torch.equal(oq, q_ref) and torch.equal(so.view(torch.int32), s_ref.view(torch.int32)), rep


def test_fp8_output_chains_two_large_layers(orc):
    # layer a (panel kernel, FP8 out) feeds layer b directly: same bits as bf16 hand-over + loka_quantize
    M, K, H, N = 1024, 512, 2048, 1024
    x = synth.student_t4(M, K, seed=31)
    w1, w2 = synth.weight(K, H, seed=32), synth.weight(H, N, seed=33)
    xq, sx = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
    w1q, s1 = B.loka_quantize(w1.to(DEV), B.SCALE_COL, transpose_out=True)
    w2q, s2 = B.loka_quantize(w2.to(DEV), B.SCALE_COL, transpose_out=True)
    v = B.variant_id("panel32_256x256")
    da = B.make_desc(M, H, K, 1, norm=B.NORM_LAYERNORM, variant=v)
    db = B.make_desc(M, N, H, 1, norm=B.NORM_RMSNORM, variant=v)
    hq, hs, _ = B.loka_fp8_gemm_norm_fp8out(da, xq, sx, w1q, s1)
    out_fused, _ = B.loka_fp8_gemm_norm(db, hq, hs, w2q, s2)
    h, _ = B.loka_fp8_gemm_norm(da, xq, sx, w1q, s1)
    hq2, hs2 = B.loka_quantize(h, B.SCALE_ROW)
    out_ref, _ = B.loka_fp8_gemm_norm(db, hq2, hs2, w2q, s2)
    torch.cuda.synchronize()
    assert torch.equal(hq, hq2) and torch.equal(hs, hs2)
    assert torch.equal(out_fused.view(torch.int16), out_ref.view(torch.int16))
    hq_o, hs_o = orc.quantize(to_np_bits(h), orc.SCALE_ROW)
    assert np.array_equal(hq.cpu().numpy(), hq_o) and np.array_equal(hs.cpu().numpy().view(np.uint32), hs_o.view(np.uint32))


@pytest.mark.parametrize("shape", [(2048, 512, 2048), (1000, 256, 256), (3000, 256, 1024), (600, 2048, 512)])
def test_fp8_output_with_the_library_choice(orc, shape):
    # variant -1: whichever kernel the library picks must deliver codes and scales that decode to the bf16 output of
    # the plain call within the e4m3 step (half a step of 2^-3 relative to the row amax, plus the kernels' own
    # last-bit differences)
    M, K, N = shape
    x, wt = synth.normal(M, K, seed=41).to(DEV), synth.weight(K, N, seed=42).to(DEV)
    xq, sx = B.loka_quantize(x, B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt, B.SCALE_COL, transpose_out=True)
    desc = B.make_desc(M, N, K, 1, norm=B.NORM_LAYERNORM)
    out, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw)
    torch.cuda.synchronize()
    dec = oq.view(torch.float8_e4m3fn).float() * so[:, None]
    amax = out.float().abs().amax(dim=1, keepdim=True)
    assert torch.equal(so, torch.clamp(amax[:, 0], min=1e-12) / 448.0) or torch.allclose(so, amax[:, 0] / 448.0, rtol=2e-2)
    assert bool(((dec - out.float()).abs() <= amax * (2.0 ** -4 + 2.0 ** -6)).all())
    # the oracle's quantization of the plain call's bf16 output: same scales up to the two kernels' last-bit
    # differences in the row's largest value, and codes at most one e4m3 step apart where those differences cross a
    # rounding boundary (bit-exact when the library picks the same kernel for both calls)
    q_o, s_o = orc.quantize(to_np_bits(out), orc.SCALE_ROW)
    assert np.allclose(so.cpu().numpy(), s_o, rtol=2.0 ** -6, atol=0)
    dec_o = torch.from_numpy(q_o).view(torch.float8_e4m3fn).float() * torch.from_numpy(s_o)[:, None]
    assert bool(((dec.cpu() - dec_o).abs() <= amax.cpu() * 2.0 ** -4).all())
    if np.array_equal(so.cpu().numpy().view(np.uint32), s_o.view(np.uint32)):
        assert (oq.cpu().numpy() != q_o).mean() < 1e-3


def test_fp8_output_unsupported_cases():
    M, K, N = 512, 4096, 4096                                                 # rows wider than a workgroup keeps
    xq, sx = torch.zeros(M, K, dtype=torch.uint8, device=DEV), torch.ones(M, device=DEV)
    wq, sw = torch.zeros(N, K, dtype=torch.uint8, device=DEV), torch.ones(N, device=DEV)
    # the panel kernel's FP8 output needs a row norm (LayerNorm / RMSNorm)
    with pytest.raises(B.LokaError):
        B.loka_fp8_gemm_norm_fp8out(B.make_desc(M, N, K, 1, norm=B.NORM_NONE), xq, sx, wq, sw)
    # a tiled variant without the epilogue
    with pytest.raises(B.LokaError):
        B.loka_fp8_gemm_norm_fp8out(B.make_desc(M, N, K, 1, variant=B.variant_id("twopass128x128")), xq, sx, wq, sw)


# ----------------------------------------------------------------------------- backward-pass GEMMs through the same entry points
@pytest.mark.parametrize("shape", [(512, 256, 384), (1024, 512, 256)])
def test_backward_gemms_with_the_forward_entry_points(orc, shape):
    # dX = dY . W^T and dW = X^T . dY (Section 3.3: forward and backward GEMMs are routed separately): both are
    # "rows times K-contiguous rows" products once the operands are quantized in the right orientation
    M, K, N = shape
    x = synth.normal(M, K, seed=3 * M)
    w = synth.weight(K, N, seed=3 * N)
    dy = synth.normal(M, N, seed=3 * K, std=0.02)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)

    # dX [M, K]: contraction over N.  dY rowwise; W [K, N] quantized as it lies (one scale per row k = per output column)
    dyq, sdy = B.loka_quantize(dyd, B.SCALE_ROW)
    wq, sw = B.loka_quantize(wd, B.SCALE_ROW)
    d1 = B.make_desc(M, K, N, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_NONE)
    _, dx = B.loka_fp8_gemm_norm(d1, dyq, sdy, wq, sw, want_y=True)
    dyq_o, sdy_o = orc.quantize(synth.bf16_bits(dy), B.SCALE_ROW)
    wq_o, sw_o = orc.quantize(synth.bf16_bits(w), B.SCALE_ROW)
    assert np.array_equal(dyq.cpu().numpy(), dyq_o) and np.array_equal(wq.cpu().numpy(), wq_o)
    dx_o, ad = orc.fp8_gemm(dyq_o, sdy_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, want_absdot=True)
    check_fp32_y(dx.cpu().numpy(), dx_o, ad, dyq_o, sdy_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, N, "dX")
    ref = dy.double() @ w.double().T                                        # sanity against the unquantized product
    assert rel_fro(dx.cpu().numpy(), ref.numpy()) < 0.06

    # dW [K, N]: contraction over M.  X and dY quantized per column and written transposed ([K, M], [N, M])
    xtq, sxt = B.loka_quantize(xd, B.SCALE_COL, transpose_out=True)
    dytq, sdyt = B.loka_quantize(dyd, B.SCALE_COL, transpose_out=True)
    d2 = B.make_desc(K, N, M, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_NONE)
    _, dw = B.loka_fp8_gemm_norm(d2, xtq, sxt, dytq, sdyt, want_y=True)
    xtq_o, sxt_o = orc.quantize(synth.bf16_bits(x), B.SCALE_COL, transpose_out=True)
    dytq_o, sdyt_o = orc.quantize(synth.bf16_bits(dy), B.SCALE_COL, transpose_out=True)
    assert np.array_equal(xtq.cpu().numpy(), xtq_o) and np.array_equal(dytq.cpu().numpy(), dytq_o)
    dw_o, ad = orc.fp8_gemm(xtq_o, sxt_o, B.SCALE_ROW, dytq_o, sdyt_o, B.SCALE_COL, want_absdot=True)
    check_fp32_y(dw.cpu().numpy(), dw_o, ad, xtq_o, sxt_o, B.SCALE_ROW, dytq_o, sdyt_o, B.SCALE_COL, M, "dW")
    ref = x.double().T @ dy.double()
    assert rel_fro(dw.cpu().numpy(), ref.numpy()) < 0.06


@pytest.mark.parametrize("shape", [(1024, 256, 384), (4096, 512, 512), (65536, 256, 1024)])
def test_weight_gradient_with_block_scales_along_the_batch(orc, shape):
    # dW = X^T dY with the block recipe: the contraction runs over the batch rows, so the scale groups do too.  X is
    # quantized BLOCK_128x1 and dY BLOCK_128x128, both in ONE pass with the output transposed; the GEMM is the forward
    # entry point with (M', N', K') = (K, N, M), which the library runs split over K (few output tiles, long K).
    M, K, N = shape
    x = synth.normal(M, K, seed=2 * M + 1)
    dy = synth.normal(M, N, seed=2 * N + 1, std=0.02)
    dy[:, 5] *= 300.0                                        # one channel of the gradient with outliers
    xtq, sxt = B.loka_quantize(x.to(DEV), B.SCALE_BLOCK_128x1, transpose_out=True)          # [K, M], [K, M/128]
    dytq, sdyt = B.loka_quantize(dy.to(DEV), B.SCALE_BLOCK_128x128, transpose_out=True)     # [N, M], [M/128, N/128]
    d = B.make_desc(K, N, M, 1, B.SCALE_BLOCK_1x128, B.SCALE_BLOCK_128x128, B.NORM_NONE)
    if M >= 2048:
        assert B.loka_variant_name(B.loka_default_variant(d)) == "splitk128x128"
    out, dw = B.loka_fp8_gemm_norm(d, xtq, sxt, dytq, sdyt, want_y=True)
    torch.cuda.synchronize()
    xtq_o, sxt_o = orc.quantize(synth.bf16_bits(x), orc.SCALE_BLOCK_128x1, transpose_out=True)
    dytq_o, sdyt_o = orc.quantize(synth.bf16_bits(dy), orc.SCALE_BLOCK_128x128, transpose_out=True)
    assert np.array_equal(xtq.cpu().numpy(), xtq_o) and np.array_equal(sxt.cpu().numpy().view(np.uint32), sxt_o.view(np.uint32))
    assert np.array_equal(dytq.cpu().numpy(), dytq_o) and np.array_equal(sdyt.cpu().numpy().view(np.uint32), sdyt_o.view(np.uint32))
    rows = np.unique(np.linspace(0, K - 1, 24).round().astype(int))      # sampled rows of dW
    sx_sel = sxt_o.reshape(K, M // 128)[rows].ravel()
    dw_o, ad = orc.fp8_gemm(np.ascontiguousarray(xtq_o[rows]), sx_sel, orc.SCALE_BLOCK_1x128, dytq_o, sdyt_o,
                            orc.SCALE_BLOCK_128x128, want_absdot=True)
    idx = torch.from_numpy(rows).to(DEV)
    fig = check_fp32_y(dw[idx].cpu().numpy(), dw_o, ad, xtq_o[rows], sx_sel, B.SCALE_BLOCK_1x128, dytq_o, sdyt_o,
                       B.SCALE_BLOCK_128x128, M, f"dW {shape}")
    fig.pop("err")
    print("dW", shape, fig)
    assert torch.equal(out[idx].view(torch.int16), dw[idx].to(torch.bfloat16).view(torch.int16))     # bf16 O = rounding of Y
    ref = (x.double().T @ dy.double())[rows]                                # sanity against the unquantized product
    assert rel_fro(dw[idx].cpu().numpy(), ref.numpy()) < 0.05


@pytest.mark.parametrize("recipe", ["row", "block", "block_pow2", "tensor"])
def test_c5_full_size(orc, recipe):
    w = synth.WORKLOADS["C5"]
    x, wt = synth.activations(w), synth.weights(w)
    desc = B.make_desc(w.M, w.N, w.K, 1, *RECIPES[recipe], B.NORM_LAYERNORM)
    rows = _sample_rows(w.M, 48)
    if recipe == "tensor":
        x = x[:4096].contiguous()                   # the oracle quantizes the whole tensor for this recipe
        rows = _sample_rows(4096, 48)
    for v in _variants_for(desc):
        if recipe != "row" and v != B.loka_default_variant(desc):
            continue
        r = _run_case(orc, x, wt, recipe, "layernorm", v, rows=rows, tag=f"C5 {recipe} {B.loka_variant_name(v)}",
                      fro_cap=FRO_CAP["C5 " + recipe])
        print("C5", recipe, B.loka_variant_name(v), r)


def test_repeatable_bits():
    # same inputs, 10 launches: identical output bits (catches LDS races / missing barriers)
    w = synth.WORKLOADS["C2"]
    x, wt = synth.activations(w, rows=2048).to(DEV), synth.weights(w).to(DEV)
    xq, sx = B.loka_quantize(x, B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt, B.SCALE_COL, transpose_out=True)
    for v in range(B.loka_variant_count()):
        desc = B.make_desc(2048, w.N, w.K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, variant=v)
        if not B.loka_variant_supports(desc, v):
            continue
        ref, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
        for _ in range(10):
            o, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
            assert torch.equal(o.view(torch.int16), ref.view(torch.int16)), B.loka_variant_name(v)


# ----------------------------------------------------------------------------- BF16 reference GEMM
@pytest.mark.parametrize("shape", [(256, 128, 128), (300, 192, 272), (1024, 512, 512),
                                   (200, 72, 144), (130, 1000, 64), (80, 8, 16)])       # K a multiple of 8 only
def test_bf16_reference_gemm(orc, shape):
    M, K, N = shape
    x = synth.student_t4(M, K, seed=M + 1)
    wt = synth.weight(K, N, seed=N + 1)
    desc = B.make_desc(M, N, K, 1, norm=B.NORM_NONE)
    y = B.loka_bf16_gemm(desc, x.to(DEV), wt.to(DEV)).cpu().numpy()
    y_o = orc.ref_gemm(synth.bf16_bits(x), synth.bf16_bits(wt))
    absdot = (x.double().abs() @ wt.double().abs()).numpy()
    # exact bf16 products, fp32 accumulation in K/32 MFMA steps
    tol = (K / 32 + 8) * 2.0 ** -24 * absdot + 2.0 ** -23 * np.abs(y_o)
    assert (np.abs(y.astype(np.float64) - y_o) <= tol).all()
    assert rel_fro(y, y_o) <= 1e-5


def test_bf16_reference_gemm_grouped(orc):
    G, M, K, N = 3, 200, 128, 144
    x = synth.normal(G * M, K, seed=1)
    wt = synth.weight(G * K, N, seed=2)
    desc = B.make_desc(M, N, K, G, norm=B.NORM_NONE)
    y = B.loka_bf16_gemm(desc, x.to(DEV), wt.to(DEV)).cpu().numpy()
    for g in range(G):
        y_o = orc.ref_gemm(synth.bf16_bits(x[g * M:(g + 1) * M]), synth.bf16_bits(wt[g * K:(g + 1) * K]))
        assert rel_fro(y[g * M:(g + 1) * M], y_o) <= 1e-5


def test_bounded_wait_is_reported():
    # the panel-synchronous variants wait for the other tiles of a row panel; a wait that runs out marks the launch in
    # the workspace, the tile's rows leave as NaN, and the kernel still ends.  Forced from the host: with a limit of
    # zero polls the launch also looks for an arrival value nobody writes, so every wait runs out whatever the timing.
    M, K, N = 2048, 256, 2048
    x, wt = synth.normal(M, K, 3).to(DEV), synth.weight(K, N, 4).to(DEV)
    xq, sx = B.loka_quantize(x, B.SCALE_ROW)
    wq, sw = B.loka_quantize(wt, B.SCALE_COL, transpose_out=True)
    for vname in ("panel32_256x256", "panel256x256w8"):
        desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5, variant=B.variant_id(vname))
        # uninitialised workspace contents must not matter: fill it with a pattern first
        ws = torch.full((B.lib().loka_fp8_gemm_norm_workspace(ctypes.byref(desc)),), 0xA5, dtype=torch.uint8, device=DEV)
        good, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, workspace=ws)
        assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
        assert not bool(torch.isnan(good.float()).any())
        try:
            B.loka_test_set_spin_limit(0)
            bad, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, workspace=ws)
            assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_ERR_TIMEOUT
            assert bool(torch.isnan(bad.float()).all())              # nobody can take that launch's output for a result
        finally:
            B.loka_test_set_spin_limit(-1)
        again, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, workspace=ws)
        assert B.loka_fp8_gemm_norm_check(desc, ws) == B.LOKA_OK
        assert torch.equal(good, again)
        if vname == "panel32_256x256":
            good32 = good
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5, variant=B.variant_id("panel32_256x256"))
    # the FP8-output form of the same kernel reports through its own workspace
    ws_f = torch.full((B.lib().loka_fp8_gemm_norm_fp8out_workspace(ctypes.byref(desc)),), 0x5A, dtype=torch.uint8, device=DEV)
    gamma, beta = (t.to(DEV) for t in synth.affine(N, seed=8))
    try:
        B.loka_test_set_spin_limit(0)
        _, so_bad, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, workspace=ws_f)
        assert B.loka_fp8_gemm_norm_check(desc, ws_f) == B.LOKA_ERR_TIMEOUT
        assert bool(torch.isnan(so_bad).all())                       # FP8 output: the row scales say so
        _, so_bad2, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, gamma, beta, workspace=ws_f)   # two bounded waits per tile
        assert B.loka_fp8_gemm_norm_check(desc, ws_f) == B.LOKA_ERR_TIMEOUT
        assert bool(torch.isnan(so_bad2).all())
    finally:
        B.loka_test_set_spin_limit(-1)
    oq, so, _ = B.loka_fp8_gemm_norm_fp8out(desc, xq, sx, wq, sw, workspace=ws_f)
    assert B.loka_fp8_gemm_norm_check(desc, ws_f) == B.LOKA_OK
    q_ref, s_ref = B.loka_quantize(good32, B.SCALE_ROW)
    assert torch.equal(oq, q_ref) and torch.equal(so, s_ref)
    # a workspace that no launch has used yet has nothing to report
    fresh = torch.zeros_like(ws_f)
    assert B.loka_fp8_gemm_norm_check(desc, fresh) == B.LOKA_OK
    # variants without a cross-workgroup wait have nothing to report
    row = B.make_desc(256, 128, 128, variant=B.variant_id("row64x128"))
    assert B.loka_fp8_gemm_norm_check(row, None) == B.LOKA_OK


def test_dispatch_drops_a_candidate_whose_wait_ran_out():
    # the profiler must not time or probe a launch that produced nothing: with every wait forced to run out, the
    # panel-synchronous candidates disappear from the table and the choice falls on a kernel without such a wait
    M, K, N = 1024, 256, 1024
    x, wt = synth.normal(M, K, 5).to(DEV), synth.weight(K, N, 6).to(DEV)
    shape = B.make_desc(M, N, K, 1, norm=B.NORM_LAYERNORM)
    B.loka_dispatch_clear()
    st, ch, table = B.loka_dispatch(shape, x, wt, 5e-2)
    names = {r["variant_name"] for r in table}
    assert st == B.LOKA_OK and "panel32_256x256" in names
    B.loka_dispatch_clear()
    try:
        B.loka_test_set_spin_limit(0)
        st2, ch2, table2 = B.loka_dispatch(shape, x, wt, 5e-2)
    finally:
        B.loka_test_set_spin_limit(-1)
        B.loka_dispatch_clear()
    names2 = {r["variant_name"] for r in table2}
    assert st2 == B.LOKA_OK and not (names2 & {"panel32_256x256", "panel256x256w8"}) and names2
    assert ch2["variant_name"] in names2


# ----------------------------------------------------------------------------- quantization fused into the layer
@pytest.mark.parametrize("case", [(300, 256, 256, 1, "rmsnorm"), (1000, 128, 256, 1, "layernorm"), (77, 512, 256, 1, "layernorm"),
                                  (513, 256, 512, 1, "rmsnorm"), (260, 128, 1024, 1, "layernorm"), (640, 256, 256, 5, "rmsnorm"),
                                  (130, 128, 512, 3, "none"),
                                  # several strips per wave: the next strip's prefetch in all its forms (8 waves early,
                                  # 8 waves piecewise from inside the epilogue, 4 waves)
                                  (70000, 256, 128, 1, "layernorm"), (70000, 128, 256, 1, "rmsnorm"),
                                  (40000, 256, 256, 1, "layernorm"), (36000, 512, 128, 1, "rmsnorm")])
@pytest.mark.parametrize("variant", ["wreg32", "strip32"])
def test_fused_quantization_gives_the_bits_of_the_two_calls(orc, case, variant):
    # loka_fp8_linear_norm = loka_quantize(ROW) + loka_fp8_gemm_norm in one kernel: scales, fp32 Y and bf16 O must be
    # identical bit for bit (same codes, same kernel arithmetic); the two-call path is checked against the oracle above,
    # and the scales here against the oracle directly
    M, K, N, G, norm = case
    probe = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=B.variant_id(variant))
    if not B.loka_variant_supports(probe, B.variant_id(variant)):
        pytest.skip(f"{variant} does not cover this shape")
    x = torch.cat([synth.student_t4(M, K, 50 + g) for g in range(G)], 0)
    w = torch.cat([synth.weight(K, N, 60 + g) for g in range(G)], 0)
    gamma, beta = synth.affine(N, 9)
    xd, wd = x.to(DEV), w.to(DEV)
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s_ = B.loka_quantize(wd[g * K:(g + 1) * K], B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s_
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=B.variant_id(variant))
    xq, sx = B.loka_quantize(xd, B.SCALE_ROW)
    o2, y2 = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True)
    o1, y1, sx1 = B.loka_fp8_linear_norm(desc, xd, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True, want_sx=True)
    torch.cuda.synchronize()
    _, sx_o = orc.quantize(synth.bf16_bits(x), orc.SCALE_ROW)
    assert np.array_equal(sx1.cpu().numpy().view(np.uint32), sx_o.view(np.uint32)), "row scales differ from the oracle's"
    assert torch.equal(sx1, sx)
    assert torch.equal(y1, y2), "fp32 Y differs from the two-call path"
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), "bf16 O differs from the two-call path"


@pytest.mark.parametrize("case", [
    (16384, 512, 512, 1, "rmsnorm", "wreg32"),       # C2
    (8192 + 40, 256, 1024, 1, "layernorm", "wreg32"),  # the C3a layer, ragged last block
    (4096 + 8, 1024, 256, 1, "layernorm", "wreg32"),   # the C3b layer
    (1000, 128, 256, 1, "none", "wreg32"),
    (2048 + 16, 256, 256, 3, "rmsnorm", "wreg32"),     # grouped: a workgroup's rows cross problems
    (520, 512, 128, 5, "layernorm", "wreg32"),
    # the large-tile kernel where a tile spans the output row: 1, 2 and 4 loads of a wave per row of X
    (65536 + 72, 1024, 256, 1, "layernorm", "panel32_256x256"),   # the C3b layer and a ragged last tile; two tiles per workgroup
    (3000, 512, 128, 1, "rmsnorm", "panel32_256x256"),
    (1500, 2048, 256, 3, "layernorm", "panel32_256x256"),         # grouped
    (256 * 300 + 8, 512, 256, 1, "none", "panel32_256x256"),      # more tiles than workgroups: several tiles each
], ids=lambda c: "x".join(str(v) for v in c))
def test_quantize_prologue_gives_the_bits_of_the_two_calls(orc, case):
    # loka_fp8_linear_norm_xq: every workgroup quantizes the rows it consumes, then runs the kernel of
    # loka_fp8_gemm_norm: codes and row scales must be the oracle's (every row), fp32 Y and bf16 O those of the two calls,
    # which are checked against the oracle elsewhere in this file
    M, K, N, G, norm, vname = case
    v = B.variant_id(vname)
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=v)
    assert B.loka_variant_supports(desc, v)
    x = torch.cat([synth.student_t4(M, K, 150 + g) for g in range(G)], 0)
    x[3] = 0                                                     # an all-zero row: the amax floor
    x[M - 1, 7] = 3.0e4                                          # an outlier in the last row of the first problem
    w = torch.cat([synth.weight(K, N, 160 + g) for g in range(G)], 0)
    gamma, beta = synth.affine(N, 19)
    xd, wd = x.to(DEV), w.to(DEV)
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s_ = B.loka_quantize(wd[g * K:(g + 1) * K], B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s_
    xq2, sx2 = B.loka_quantize(xd, B.SCALE_ROW)
    o2, y2 = B.loka_fp8_gemm_norm(desc, xq2, sx2, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True)
    # output buffers pre-filled: every byte must be written by the call
    xq1 = torch.full((G * M, K), 0x5A, dtype=torch.uint8, device=DEV)
    sx1 = torch.full((G * M,), -1.0, dtype=torch.float32, device=DEV)
    for rep in range(2):                                         # (the second call finds its own codes in place)
        o1, y1, _, _ = B.loka_fp8_linear_norm_xq(desc, xd, wq, sw, gamma.to(DEV), beta.to(DEV), want_y=True, xq=xq1, sx=sx1)
        torch.cuda.synchronize()
        xq_o, sx_o = orc.quantize(synth.bf16_bits(x), orc.SCALE_ROW)
        assert np.array_equal(xq1.cpu().numpy(), xq_o), "codes differ from the oracle's"
        assert np.array_equal(sx1.cpu().numpy().view(np.uint32), sx_o.view(np.uint32)), "row scales differ from the oracle's"
        assert torch.equal(y1, y2), "fp32 Y differs from the two-call path"
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), "bf16 O differs from the two-call path"
    # (no kernel named: the library's choice for the shape where that kernel has the prologue; the bits are those of the
    # two calls on the same kernel)
    d_def = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=-1)
    o3, _, xq3, sx3 = B.loka_fp8_linear_norm_xq(d_def, xd, wq, sw, gamma.to(DEV), beta.to(DEV))
    v_def = B.loka_default_variant(d_def)
    if B.loka_variant_name(v_def) in ("wreg32", "panel32_256x256"):
        d_pin = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=v_def)
        o4, _ = B.loka_fp8_gemm_norm(d_pin, xq2, sx2, wq, sw, gamma.to(DEV), beta.to(DEV))
        assert torch.equal(o3.view(torch.int16), o4.view(torch.int16))
    assert torch.equal(xq3, xq2) and torch.equal(sx3, sx2)


def test_quantize_prologue_unsupported():
    x = torch.zeros(512, 4096, dtype=torch.bfloat16, device=DEV)
    wq = torch.zeros(4096, 4096, dtype=torch.uint8, device=DEV)
    sw = torch.ones(4096, dtype=torch.float32, device=DEV)
    with pytest.raises(B.LokaError) as e:                        # a layer the streaming kernel does not cover
        B.loka_fp8_linear_norm_xq(B.make_desc(512, 4096, 4096, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5), x, wq, sw)
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED
    x = torch.zeros(512, 256, dtype=torch.bfloat16, device=DEV)
    wq = torch.zeros(256, 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.LokaError) as e:                        # per-tensor activation scale: no row-local amax
        B.loka_fp8_linear_norm_xq(B.make_desc(512, 256, 256, 1, B.SCALE_TENSOR, B.SCALE_TENSOR, B.NORM_LAYERNORM, 1e-5), x, wq,
                                  torch.ones(1, device=DEV))
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED
    with pytest.raises(B.LokaError) as e:                        # another kernel named
        B.loka_fp8_linear_norm_xq(B.make_desc(512, 256, 256, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5,
                                              variant=B.variant_id("strip32")), x, wq, torch.ones(256, device=DEV))
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED


def test_fused_quantization_unsupported_shapes():
    # the configurations whose weights fill the register file (streaming kernel) or whose raw strip would (strip
    # kernel, K = 1024), and everything neither kernel covers
    for M, K, N in [(4096, 512, 512), (4096, 256, 1024), (4096, 1024, 256), (4096, 4096, 4096)]:
        desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, 1e-5)
        x = torch.zeros(M, K, dtype=torch.bfloat16, device=DEV)
        wq = torch.zeros(N, K, dtype=torch.uint8, device=DEV)
        sw = torch.ones(N, dtype=torch.float32, device=DEV)
        with pytest.raises(B.LokaError) as e:
            B.loka_fp8_linear_norm(desc, x, wq, sw)
        assert e.value.status == B.LOKA_ERR_UNSUPPORTED
    tens = B.make_desc(256, 256, 256, 1, B.SCALE_TENSOR, B.SCALE_TENSOR, B.NORM_LAYERNORM, 1e-5)
    with pytest.raises(B.LokaError) as e:
        B.loka_fp8_linear_norm(tens, torch.zeros(256, 256, dtype=torch.bfloat16, device=DEV),
                               torch.zeros(256, 256, dtype=torch.uint8, device=DEV), torch.ones(1, device=DEV))
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED


@pytest.mark.parametrize("variant", ["wreg32", "strip32", None])
def test_fused_quantization_c4_full_size(orc, variant):
    # the grouped workload at full size: identical bits to the two calls on every row, and sampled rows of two
    # groups against the oracle
    w = synth.WORKLOADS["C4"]
    G = w.batch
    xs = torch.cat([synth.activations(w, g) for g in range(G)], 0)
    ws = torch.cat([synth.weights(w, g) for g in range(G)], 0)
    xd, wd = xs.to(DEV), ws.to(DEV)
    wq = torch.empty(G * w.N, w.K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * w.N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s_ = B.loka_quantize(wd[g * w.K:(g + 1) * w.K], B.SCALE_COL, transpose_out=True)
        wq[g * w.N:(g + 1) * w.N] = q
        sw[g * w.N:(g + 1) * w.N] = s_
    # (no variant named: both entry points pick the strip kernel for this shape)
    desc = B.make_desc(w.M, w.N, w.K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM,
                       variant=-1 if variant is None else B.variant_id(variant))
    if variant is None:
        assert B.loka_variant_name(B.loka_default_variant(desc)) == "strip32"
    xq, sx = B.loka_quantize(xd, B.SCALE_ROW)
    o2, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
    o1, y1, sx1 = B.loka_fp8_linear_norm(desc, xd, wq, sw, want_y=True, want_sx=True)
    torch.cuda.synchronize()
    assert torch.equal(sx1, sx) and torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    for g in (0, 63):
        rows = _sample_rows(w.M, 48)
        xq_o, sx_o = orc.quantize(synth.bf16_bits(xs[g * w.M:(g + 1) * w.M])[rows].copy(), B.SCALE_ROW)
        wq_o, sw_o = orc.quantize(synth.bf16_bits(ws[g * w.K:(g + 1) * w.K]), B.SCALE_COL, transpose_out=True)
        y_o, absdot = orc.fp8_gemm(xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, want_absdot=True)
        idx = torch.from_numpy(rows + g * w.M).to(DEV)
        assert np.array_equal(sx1[idx].cpu().numpy().view(np.uint32), sx_o.view(np.uint32))
        err = check_fp32_y(y1[idx].cpu().numpy(), y_o, absdot, xq_o, sx_o, B.SCALE_ROW, wq_o, sw_o, B.SCALE_COL, w.K,
                           f"group {g}", 2.8e-5)["err"]
        ok, worst, _ = check_bf16_out(to_np_bits(o1[idx]), orc.norm(y_o, B.NORM_RMSNORM),
                                      abs_tol=propagated_abs_tol(y_o, err, B.NORM_RMSNORM, 1e-5))
        assert ok, f"group {g}: worst {worst} ulps"
