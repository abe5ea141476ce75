"""GPU parity of loka_probe_error and behaviour of loka_dispatch."""
import math

import numpy as np
import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# fp64 sums of n same-sign terms, only the summation order differs from the oracle's: each side is within
# (n-1) * 2^-53 of the exact sum, so the two agree to n * 2^-52 relative.  MERE divides with a 1-ulp fp32
# reciprocal, so its tolerance is 2^-21 relative.
REL_MERE = 2.0 ** -21


def _cmp_probe(orc, y, yref):
    st_o, rm_o = orc.probe(y, yref)
    st_g, rm_g = B.loka_probe_error(torch.from_numpy(y).to(DEV), torch.from_numpy(yref).to(DEV))
    assert np.array_equal(rm_g.cpu().numpy().view(np.uint32), rm_o.view(np.uint32)), "rowmax must be bit-exact"
    assert st_g["max_abs"] == st_o["max_abs"]
    rel_sum = max(1e-13, y.size * 2.0 ** -52)
    for k in ("sum_sq_err", "sum_sq_ref", "rel_fro"):
        assert math.isclose(st_g[k], st_o[k], rel_tol=rel_sum, abs_tol=0.0), (k, st_g[k], st_o[k])
    assert math.isclose(st_g["mere"], st_o["mere"], rel_tol=REL_MERE), (st_g["mere"], st_o["mere"])
    return st_g


@pytest.mark.parametrize("shape", [(1, 16), (7, 64), (256, 128), (1000, 272), (513, 1024), (300, 4096), (33, 12288)])
def test_probe_shapes(orc, shape):
    M, N = shape
    rng = np.random.default_rng(M * 7 + N)
    yref = rng.standard_normal((M, N)).astype(np.float32)
    y = (yref * (1 + 0.03 * rng.standard_normal((M, N)))).astype(np.float32)
    yref[0, 0] = 0.0                                          # floored denominator path
    _cmp_probe(orc, y, yref)


def test_probe_identical_inputs_and_repeatability(orc):
    rng = np.random.default_rng(0)
    yref = rng.standard_normal((4096, 512)).astype(np.float32)
    st = _cmp_probe(orc, yref.copy(), yref)
    assert st["rel_fro"] == 0 and st["max_abs"] == 0 and st["mere"] == 0
    y = torch.from_numpy((yref + 0.01 * rng.standard_normal(yref.shape)).astype(np.float32)).to(DEV)
    r = torch.from_numpy(yref).to(DEV)
    first, _ = B.loka_probe_error(y, r)
    for _ in range(5):
        again, _ = B.loka_probe_error(y, r)
        assert again == first                                 # fixed combination order: identical bits


def test_probe_of_the_fp8_path_full_c2(orc):
    # whole path on the GPU at C2's full size, probe compared with the oracle's probe of the same Y / Yref
    w = synth.WORKLOADS["C2"]
    x, wt = synth.activations(w).to(DEV), synth.weights(w).to(DEV)
    for xm, wm in ((B.SCALE_ROW, B.SCALE_COL), (B.SCALE_TENSOR, B.SCALE_TENSOR)):
        xq, sx = B.loka_quantize(x, xm)
        wq, sw = B.loka_quantize(wt, wm, transpose_out=True)
        desc = B.make_desc(w.M, w.N, w.K, 1, xm, wm, B.NORM_RMSNORM)
        _, y = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, want_y=True)
        yref = B.loka_bf16_gemm(desc, x, wt)
        st = _cmp_probe(orc, y.cpu().numpy(), yref.cpu().numpy())
        assert 0.02 < st["rel_fro"] < 0.06                    # e4m3: a few 1e-2 whatever the recipe
        print("C2 probe", xm, wm, st)


def test_dispatch_select_matches_oracle_rule(orc):
    rng = np.random.default_rng(3)
    for _ in range(200):
        n = int(rng.integers(1, 9))
        usec = rng.uniform(1, 20, n)
        err = rng.uniform(0, 0.06, n)
        budget = float(rng.uniform(0, 0.06))
        floor = float(rng.choice([0.0, 1.05, 1.5]))
        base = float(rng.uniform(5, 25))
        assert B.loka_dispatch_select(usec, err, budget, floor, base) == orc.dispatch_select(usec, err, budget, floor, base)


def test_dispatch_small_shape_budgets_and_cache():
    w = synth.WORKLOADS["C1"]
    x, wt = synth.activations(w).to(DEV), synth.weights(w).to(DEV)
    desc = B.make_desc(w.M, w.N, w.K, 1, norm=B.NORM_LAYERNORM)
    B.loka_dispatch_clear()
    # e4m3's rel-Frobenius error is a few 1e-2: a 1e-3 budget admits nothing -> stay in BF16
    st, ch, table = B.loka_dispatch(desc, x, wt, 1e-3)
    assert st == B.LOKA_ERR_NO_CANDIDATE and ch["variant"] == -1 and not ch["from_cache"]
    assert len(table) >= 3 and not any(r["feasible"] for r in table)
    assert all(0.01 < r["stats"]["rel_fro"] < 0.08 for r in table)
    # generous budget: the fastest candidate of the table is returned
    st, ch, table = B.loka_dispatch(desc, x, wt, 0.1)
    assert st == B.LOKA_OK and all(r["feasible"] for r in table)
    best = min(table, key=lambda r: r["usec"])
    assert (ch["x_mode"], ch["w_mode"], ch["variant"]) == (best["x_mode"], best["w_mode"], best["variant"])
    # same key again: answered from the cache, same choice
    st2, ch2, _ = B.loka_dispatch(desc, x, wt, 0.1)
    assert st2 == B.LOKA_OK and ch2["from_cache"] and ch2["variant"] == ch["variant"]
    # the chosen variant becomes the library's default for that shape and recipe
    d2 = B.make_desc(w.M, w.N, w.K, 1, ch["x_mode"], ch["w_mode"], B.NORM_LAYERNORM)
    assert B.loka_variant_supports(d2, B.loka_default_variant(d2))
    # an impossible speedup floor empties the feasible set as well
    st3, ch3, _ = B.loka_dispatch(desc, x, wt, 0.1, min_speedup=1e6)
    assert st3 == B.LOKA_ERR_NO_CANDIDATE and ch3["variant"] == -1


def test_dispatch_outlier_layer_prefers_finer_scales():
    # C5-like data at reduced M: blockwise scaling has the smallest error, per-tensor the largest
    w = synth.WORKLOADS["C5"]
    M = 2048
    x, wt = synth.activations(w, rows=M).to(DEV), synth.weights(w).to(DEV)
    desc = B.make_desc(M, w.N, w.K, 1, norm=B.NORM_LAYERNORM)
    B.loka_dispatch_clear()
    st, ch, table = B.loka_dispatch(desc, x, wt, 1e-2)
    assert st == B.LOKA_ERR_NO_CANDIDATE                       # 1e-2 is below what 3 mantissa bits can deliver
    err = {}
    for r in table:
        err.setdefault((r["x_mode"], r["w_mode"]), r["stats"]["rel_fro"])
    e_t = err[(B.SCALE_TENSOR, B.SCALE_TENSOR)]
    e_r = err[(B.SCALE_ROW, B.SCALE_COL)]
    e_b = err[(B.SCALE_BLOCK_1x128, B.SCALE_BLOCK_128x128)]
    print("C5-like rel_fro: tensor %.4f row %.4f block %.4f" % (e_t, e_r, e_b))
    assert e_b < e_r <= e_t * 1.05 and 0.015 < e_b < 0.06
    # a budget between blockwise and the rest admits only blockwise candidates
    mid = (e_b + min(e_r, e_t)) / 2
    st, ch, table = B.loka_dispatch(desc, x, wt, mid)
    assert st == B.LOKA_OK and ch["x_mode"] == B.SCALE_BLOCK_1x128


def test_machine_ceilings_are_plausible():
    # the measurement aid behind bench.py's "fraction of the measured ceiling": register-only matrix rates below the
    # datasheet peaks (5.0 / 2.5 PFLOP/s) but well above half of them, a copy rate below 8 TB/s and above 2
    buf = torch.empty(1 << 30, dtype=torch.uint8, device=DEV)
    f8 = B.loka_machine_ceiling(0, 20.0, buf)
    bf = B.loka_machine_ceiling(1, 20.0, buf)
    cp = B.loka_machine_ceiling(2, 10.0, buf)
    st = B.loka_machine_ceiling(3, 10.0, buf)       # operands into the LDS of every CU, no arithmetic
    print("ceilings: fp8 %.0f TFLOP/s, bf16 %.0f TFLOP/s, copy %.0f GB/s, operand stream %.0f GB/s" % (f8, bf, cp, st))
    assert 2500.0 < f8 < 5100.0 and 1250.0 < bf < 2600.0 and 2000.0 < cp < 8000.0 and 4000.0 < st < 40000.0
    f8v = B.loka_machine_ceiling(4, 20.0, buf)      # the same instructions on operands that change every instruction
    bfv = B.loka_machine_ceiling(5, 20.0, buf)
    print("ceilings with varied operands: fp8 %.0f TFLOP/s, bf16 %.0f TFLOP/s" % (f8v, bfv))
    assert 1500.0 < f8v <= f8 * 1.02 and 800.0 < bfv <= bf * 1.02
    f16c, f16v = B.loka_machine_ceiling(6, 20.0, buf), B.loka_machine_ceiling(7, 20.0, buf)     # the 16x16x128 form
    print("ceilings, 16x16x128 form: fp8 %.0f TFLOP/s on constant, %.0f on varied operands" % (f16c, f16v))
    assert 2500.0 < f16c < 5100.0 and 1500.0 < f16v <= f16c * 1.02
    with pytest.raises(B.LokaError):
        B.loka_machine_ceiling(8, 1.0, buf)
    with pytest.raises(B.LokaError):                # the operand stream needs a panel per CU and the shared matrix
        B.loka_machine_ceiling(3, 1.0, buf[:1 << 26])
