"""GPU parity of loka_tracker_update (Section 3.1, "Online Distribution Learning") against the oracle.

Tolerance.  The library evaluates S_b as X^T X - B mu_b mu_b^T with X^T X accumulated in fp32 on the
matrix cores (products of bf16 values are exact) and everything else in fp64.  n fp32 additions of terms p_m
deviate from the exact sum by at most n * 2^-23 * sum|p_m| (2^-23 per addition covers truncating adders too),
so with the oracle's magnitude A_ij = sum_m |x_mi||x_mj| + B |mu_b,i||mu_b,j|:
    |sigma_gpu - sigma_orc| <= B * 2^-23 * A_ij + 2^-23 * |sigma_orc|          (last term: the two final roundings)
mu is a fp64 column sum rounded once on both sides: <= 1 fp32 ulp.  Beside the rigorous bound the increment
must agree to 1e-6 in Frobenius norm (rounding errors average out; measured ~1e-7).
"""
import numpy as np
import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _state(K, seed):
    """A symmetric positive scatter, a mean and a row count to start from."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((K + 8, K))
    return 500, rng.uniform(-1, 1, K).astype(np.float32), (a.T @ a * 40.0).astype(np.float32)


def _step_both(orc, x, n_old, mu, sigma):
    """One update on both sides from the same state; returns (oracle mu, sigma, abs magnitude), (gpu mu, sigma)."""
    mu_o, sg_o = mu.copy(), sigma.copy()
    _, ab = orc.tracker_update(synth.bf16_bits(x), n_old, mu_o, sg_o, want_abs=True)
    mu_g = torch.from_numpy(mu.copy()).to(DEV)
    sg_g = torch.from_numpy(sigma.copy()).to(DEV)
    n_new = B.loka_tracker_update(x.to(DEV), n_old, mu_g, sg_g)
    torch.cuda.synchronize()
    assert n_new == n_old + x.shape[0]
    return (mu_o, sg_o, ab), (mu_g.cpu().numpy(), sg_g.cpu().numpy())


def _check(x, sigma_old, o, g):
    (mu_o, sg_o, ab), (mu_g, sg_g) = o, g
    rows = x.shape[0]
    ulp = np.spacing(np.abs(mu_o).astype(np.float32)).astype(np.float64)
    assert (np.abs(mu_g.astype(np.float64) - mu_o) <= ulp).all(), "mu: more than 1 fp32 ulp"
    tol = rows * 2.0 ** -23 * ab + 2.0 ** -23 * np.abs(sg_o.astype(np.float64)) + 1e-30
    d = np.abs(sg_g.astype(np.float64) - sg_o)
    worst = float((d / tol).max())
    assert worst <= 1.0, f"sigma outside the bound: {worst:.3g} x tol"
    inc_o = sg_o.astype(np.float64) - sigma_old
    rel = np.linalg.norm(sg_g.astype(np.float64) - sg_o) / max(np.linalg.norm(inc_o), 1e-300)
    assert rel <= 1e-6, f"increment rel-Frobenius {rel:.3g}"
    return worst, rel


@pytest.mark.parametrize("shape", [(64, 128), (37, 136), (1000, 136), (4096, 256), (777, 512), (5000, 392), (300, 1024)])
def test_single_update_from_a_given_state(orc, shape):
    rows, K = shape
    x = synth.correlated(rows, K, seed=rows * 31 + K)
    n_old, mu, sigma = _state(K, K + rows)
    o, g = _step_both(orc, x, n_old, mu, sigma)
    _check(x, sigma.astype(np.float64), o, g)
    assert np.array_equal(g[1], g[1].T), "symmetric state in, symmetric state out (bit for bit)"


def test_first_batch_and_constant_columns(orc):
    # from the empty state; a constant column has zero scatter: its own sum of squares is exact in fp32 and cancels
    # exactly against B mu^2 (its products with other columns round in fp32 and stay within the bound)
    K = 128
    x = synth.correlated(512, K, seed=5)
    x[:, 7] = 1.5
    x[:, 100] = -3.0
    z = np.zeros(K, np.float32), np.zeros((K, K), np.float32)
    o, g = _step_both(orc, x, 0, *z)
    _check(x, np.zeros((K, K)), o, g)
    assert g[1][7, 7] == 0 and g[1][100, 100] == 0 and g[1][7, 100] == 0 and g[0][7] == 1.5 and g[0][100] == -3.0


def test_stream_of_batches_each_side_on_its_own_state(orc):
    # three batches of different sizes and means, each side carrying its own state: the differences add up
    K = 264
    parts = [synth.correlated(1500, K, seed=1), synth.correlated(33, K, seed=2, mean_span=6.0), synth.correlated(4100, K, seed=3)]
    mu_o = np.zeros(K, np.float32); sg_o = np.zeros((K, K), np.float32)
    mu_g = torch.zeros(K, device=DEV); sg_g = torch.zeros(K, K, device=DEV)
    n_o = n_g = 0
    tol = np.zeros((K, K))
    for x in parts:
        n_o, ab = orc.tracker_update(synth.bf16_bits(x), n_o, mu_o, sg_o, want_abs=True)
        n_g = B.loka_tracker_update(x.to(DEV), n_g, mu_g, sg_g)
        # this step's own bound, plus the sensitivity of the rank-1 term to the 1-ulp difference in the carried mean
        tol += x.shape[0] * 2.0 ** -23 * ab + 2.0 ** -22 * np.abs(sg_o) + 2.0 ** -20 * np.sqrt(np.outer(np.diag(sg_o), np.diag(sg_o)))
    torch.cuda.synchronize()
    assert n_o == n_g == 5633
    assert (np.abs(mu_g.cpu().numpy().astype(np.float64) - mu_o) <= 4 * np.spacing(np.abs(mu_o))).all()
    d = np.abs(sg_g.cpu().numpy().astype(np.float64) - sg_o)
    assert (d <= tol).all(), float((d / tol).max())
    allx = torch.cat(parts, 0).double().numpy()
    c = allx - allx.mean(0)
    assert np.linalg.norm(sg_g.cpu().numpy() - c.T @ c) / np.linalg.norm(c.T @ c) < 1e-6


def test_leading_dimension_and_repeatability(orc):
    K, ld, rows = 256, 320, 2000
    big = synth.correlated(rows, ld, seed=9)
    x = big[:, :K]
    n_old, mu, sigma = _state(K, 3)
    mu_o, sg_o = mu.copy(), sigma.copy()
    orc.tracker_update(synth.bf16_bits(x.contiguous()), n_old, mu_o, sg_o)
    xg = big.to(DEV)[:, :K]                                   # a strided view: ld = 320
    outs = []
    for _ in range(3):
        mu_g = torch.from_numpy(mu.copy()).to(DEV); sg_g = torch.from_numpy(sigma.copy()).to(DEV)
        B.loka_tracker_update(xg, n_old, mu_g, sg_g)
        torch.cuda.synchronize()
        outs.append((mu_g.cpu().numpy(), sg_g.cpu().numpy()))
    assert all(np.array_equal(outs[0][0], m) and np.array_equal(outs[0][1], s) for m, s in outs[1:])
    assert np.linalg.norm(outs[0][1].astype(np.float64) - sg_o) / np.linalg.norm(sg_o.astype(np.float64) - sigma) < 1e-6


def test_large_layer_on_sampled_columns(orc):
    # C5-sized input (32768 x 4096 with outlier channels): the oracle runs on a column subset, which is
    # exactly the matching sub-block of the full summary (entry (i, j) depends on columns i and j only)
    w = synth.WORKLOADS["C5"]
    x, out_cols = synth.normal_outlier4(w.M, w.K, w.seed)
    x = x + torch.linspace(-1, 1, w.K).to(torch.bfloat16)     # non-zero column means
    rng = np.random.default_rng(0)
    cols = np.unique(np.concatenate([rng.choice(w.K, 40, replace=False), out_cols.numpy(), [0, 127, 128, 4095]]))
    mu_g = torch.zeros(w.K, device=DEV); sg_g = torch.zeros(w.K, w.K, device=DEV)
    B.loka_tracker_update(x.to(DEV), 0, mu_g, sg_g)
    torch.cuda.synchronize()
    xs = x[:, torch.from_numpy(cols)].contiguous()
    mu_o = np.zeros(len(cols), np.float32); sg_o = np.zeros((len(cols), len(cols)), np.float32)
    _, ab = orc.tracker_update(synth.bf16_bits(xs), 0, mu_o, sg_o, want_abs=True)
    sub = sg_g.cpu().numpy()[np.ix_(cols, cols)]
    _check(xs, np.zeros_like(ab), (mu_o, sg_o, ab), (mu_g.cpu().numpy()[cols], sub))
    full = sg_g.cpu().numpy()
    assert np.array_equal(full, full.T)
