"""GPU parity of loka_quantize / loka_e4m3_from_f32 against the CPU oracle: bit-exact codes and scales."""
import numpy as np
import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cmp_quant(orc, x_cpu, mode, transpose_out=False, what=""):
    xb = synth.bf16_bits(x_cpu)
    q_o, s_o = orc.quantize(xb, mode, transpose_out=transpose_out)
    q_g, s_g = B.loka_quantize(x_cpu.to(DEV), mode, transpose_out)
    torch.cuda.synchronize()
    q_g = q_g.cpu().numpy(); s_g = s_g.cpu().numpy()
    assert np.array_equal(s_g.view(np.uint32), s_o.view(np.uint32)), f"{what}: scales differ"
    nbad = int((q_g != q_o).sum())
    assert nbad == 0, f"{what}: {nbad} codes differ"


def test_hw_cast_on_every_bf16_value_and_midpoints(orc):
    # every bf16 pattern (as fp32), every e4m3 rounding midpoint and its fp32 neighbours, big magnitudes
    allb = (np.arange(65536, dtype=np.uint32) << 16).view(np.float32)
    allb = allb[np.isfinite(allb)]
    vals = [float(orc.e4m3_decode(c)) for c in range(0x7F)]
    mids = np.array([(a + b) / 2 for a, b in zip(vals, vals[1:])], dtype=np.float32)
    near = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9))])
    rng = np.random.default_rng(1)
    rnd = (rng.standard_normal(1 << 20) * np.exp(rng.uniform(-12, 7, 1 << 20))).astype(np.float32)
    t = np.concatenate([allb, near, -near, rnd, np.array([448, 449, 463.9, 464, 480, 1e6, 3e38], dtype=np.float32)])
    got = B.loka_e4m3_from_f32(torch.from_numpy(t).to(DEV)).cpu().numpy()
    want = orc.e4m3_encode_array(t)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, [(float(t[i]), hex(got[i]), hex(want[i])) for i in bad[:8]]


@pytest.mark.parametrize("mode_name", ["TENSOR", "ROW", "COL", "BLOCK_1x128", "BLOCK_128x128", "BLOCK_1x128_POW2",
                                       "BLOCK_128x128_POW2"])
@pytest.mark.parametrize("shape", [(256, 128), (384, 512), (130 * 16, 1024), (128, 4096)])
def test_modes_and_shapes(orc, mode_name, shape):
    mode = getattr(B, "SCALE_" + mode_name)
    rows, cols = shape
    if mode in (B.SCALE_BLOCK_128x128, B.SCALE_BLOCK_128x128_POW2) and rows % 128:
        rows = (rows // 128) * 128
    x = synth.student_t4(rows, cols, seed=rows + cols)
    x[3, :] = 0                       # all-zero row
    x[5, 7] = 2.0e4                   # single outlier
    x[9, :] = 448.0                   # saturating constant row
    x[11, 0:16] = torch.tensor([2.0 ** -k for k in range(16)])   # wide dynamic range incl. values that underflow
    _cmp_quant(orc, x, mode, what=f"{mode_name} {shape}")


@pytest.mark.parametrize("mode_name", ["TENSOR", "COL", "BLOCK_128x128", "BLOCK_128x128_POW2"])
def test_weight_layout_transposed(orc, mode_name):
    mode = getattr(B, "SCALE_" + mode_name)
    for K, N in ((128, 128), (512, 384), (1024, 256)):
        w = synth.weight(K, N, seed=K + N)
        _cmp_quant(orc, w, mode, transpose_out=True, what=f"{mode_name} W[{K},{N}]^T")


@pytest.mark.parametrize("shape", [(128, 16), (256, 48), (1024, 256), (4096, 1008), (65536, 256), (384, 2064)])
def test_column_blocks_for_the_weight_gradient_operands(orc, shape):
    # BLOCK_128x1 with the output transposed: the [cols, rows] codes and [cols][rows/128] scales a BLOCK_1x128 operand
    # has; one pass over the input
    rows, cols = shape
    x = synth.student_t4(rows, cols, seed=rows + cols)
    x[0:128, 3] = 0                   # an all-zero group
    x[rows - 2, 5] = 3.0e4            # a single outlier in a group
    if rows >= 256:
        x[128:256, 7] = -448.0        # a constant group
    _cmp_quant(orc, x, B.SCALE_BLOCK_128x1, transpose_out=True, what=f"128x1 {shape}")
    assert B.lib().loka_quantize_workspace(B.SCALE_BLOCK_128x1, rows, cols, 1) == 0
    assert B.lib().loka_quantize_workspace(B.SCALE_BLOCK_128x128, 256, 256, 1) == 0
    with pytest.raises(B.LokaError) as e:
        B.loka_quantize(x.to(DEV), B.SCALE_BLOCK_128x1, transpose_out=False)
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED


@pytest.mark.parametrize("cols", [16, 48, 208, 1040, 2064, 8192, 8192 + 512, 16384 + 128])
def test_ragged_and_long_rows(orc, cols):
    # widths that are not a power of two, and rows beyond the register-resident kernels
    rows = 37
    x = synth.normal(rows, cols, seed=cols)
    _cmp_quant(orc, x, B.SCALE_ROW, what=f"ROW cols={cols}")
    if cols % 128 == 0:
        _cmp_quant(orc, x, B.SCALE_BLOCK_1x128, what=f"1x128 cols={cols}")
        _cmp_quant(orc, x, B.SCALE_BLOCK_1x128_POW2, what=f"1x128 power-of-two cols={cols}")


def test_strided_input(orc):
    x = synth.normal(64, 512, seed=5)
    xd = x.to(DEV)[:, :256]                        # ld = 512 > cols = 256
    q_g, s_g = B.loka_quantize(xd, B.SCALE_ROW)
    q_o, s_o = orc.quantize(synth.bf16_bits(x[:, :256].contiguous()), B.SCALE_ROW)
    assert np.array_equal(q_g.cpu().numpy(), q_o) and np.array_equal(s_g.cpu().numpy(), s_o)


def test_workloads_full_size_rowwise(orc):
    # the activations of every benchmark configuration at full size, rowwise (sampled rows for the largest)
    for name in ("C1", "C2", "C3a", "C3b", "C4", "C5"):
        w = synth.WORKLOADS[name]
        x = synth.activations(w)
        q_g, s_g = B.loka_quantize(x.to(DEV), B.SCALE_ROW)
        torch.cuda.synchronize()
        rows = np.arange(w.M) if w.M * w.K <= (1 << 24) else np.unique(
            np.concatenate([np.arange(64), np.random.default_rng(0).integers(0, w.M, 2048), np.arange(w.M - 64, w.M)]))
        xs = synth.bf16_bits(x)[rows].copy()
        q_o, s_o = orc.quantize(xs, B.SCALE_ROW)
        idx = torch.from_numpy(rows).to(DEV)
        assert np.array_equal(q_g[idx].cpu().numpy(), q_o), name
        assert np.array_equal(s_g[idx].cpu().numpy().view(np.uint32), s_o.view(np.uint32)), name


@pytest.mark.parametrize("mode_name", ["ROW", "BLOCK_1x128", "BLOCK_1x128_POW2"])
@pytest.mark.parametrize("shape", [(1000, 256), (32768 + 24, 512), (1000, 1024), (16384 + 8, 1024), (65536 + 8, 256)])
def test_row_kernel_instances_on_both_sides_of_the_size_rule(orc, mode_name, shape):
    # the launcher gives a small tensor fewer rows per wave than a large one: both sets of instances, ragged row counts
    rows, cols = shape
    mode = getattr(B, "SCALE_" + mode_name)
    x = synth.normal(rows, cols, seed=rows + cols)
    q_g, s_g = B.loka_quantize(x.to(DEV), mode)
    torch.cuda.synchronize()
    sel = np.unique(np.concatenate([np.arange(min(rows, 130)), np.arange(rows - 130, rows), np.arange(0, rows, 257)]))
    q_o, s_o = orc.quantize(synth.bf16_bits(x)[sel].copy(), mode)
    idx = torch.from_numpy(sel).to(DEV)
    assert np.array_equal(q_g[idx].cpu().numpy(), q_o)
    s_g = s_g.cpu().numpy().reshape(rows, -1)[sel].ravel()
    assert np.array_equal(s_g.view(np.uint32), s_o.view(np.uint32))


def test_c5_recipes_full_size(orc):
    # outlier-heavy layer: per-tensor and 1x128 activations, 128x128 weights
    w = synth.WORKLOADS["C5"]
    x = synth.activations(w, rows=4096)            # same distribution, fewer rows: the oracle runs in full
    _cmp_quant(orc, x, B.SCALE_TENSOR, what="C5 tensor")
    _cmp_quant(orc, x, B.SCALE_BLOCK_1x128, what="C5 1x128")
    wt = synth.weights(w)
    _cmp_quant(orc, wt, B.SCALE_BLOCK_128x128, transpose_out=True, what="C5 W 128x128")
    _cmp_quant(orc, wt, B.SCALE_COL, transpose_out=True, what="C5 W col")


def test_argument_errors_leave_outputs_alone():
    x = torch.zeros(16, 24, dtype=torch.bfloat16, device=DEV)        # cols % 16 != 0
    with pytest.raises(B.LokaError) as e:
        B.loka_quantize(x, B.SCALE_ROW)
    assert e.value.status == B.LOKA_ERR_SHAPE
    x = torch.zeros(16, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.LokaError) as e:
        B.loka_quantize(x, B.SCALE_ROW, transpose_out=True)
    assert e.value.status == B.LOKA_ERR_UNSUPPORTED
