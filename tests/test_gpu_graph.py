"""The hot entry points under HIP graph capture.

`loka_quantize` (row / 1x128 modes), `loka_fp8_gemm_norm`, `loka_fp8_gemm_norm_fp8out` and `loka_fp8_linear_norm_xq` only launch kernels on the caller's stream (scratch comes
in as a workspace argument and is cleared by a kernel, never by a memset node), so a serving loop can record a step
once and replay it.  Each case records quantize + GEMM+norm, replays the graph several times with new activations
written into the same input buffer and eager work on the device between the replays, and compares every replay
bit for bit with the eager calls on the same input.
"""
import ctypes

import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# (M, K, N, batch, norm, what it exercises)
CASES = [
    (2048, 512, 512, 1, B.NORM_RMSNORM, "row in one tile"),
    (16384, 256, 256, 4, B.NORM_RMSNORM, "strip kernel, grouped"),
    (16384, 256, 1024, 1, B.NORM_LAYERNORM, "streaming kernel, deferred stores"),
    (4096, 256, 4096, 1, B.NORM_LAYERNORM, "panel-synchronous kernel: counters cleared by a kernel inside the launch"),
    (2048, 512, 2048, 1, B.NORM_LAYERNORM, "panel-synchronous kernel, FP8 output with gamma / beta: two exchanges per tile"),
    (8192, 256, 1024, 1, B.NORM_RMSNORM, "streaming kernel, FP8 output"),
    (8192 + 24, 512, 512, 1, B.NORM_RMSNORM, "streaming kernel, one launch: quantize prologue"),
    (2048 + 8, 256, 512, 3, B.NORM_LAYERNORM, "streaming kernel, one launch: quantize prologue, grouped"),
]


@pytest.mark.parametrize("M,K,N,G,norm,what", CASES)
def test_step_replays_from_a_graph(M, K, N, G, norm, what):
    L = B.lib()
    rows = G * M
    xs = [synth.normal(rows, K, seed=300 + i).to(DEV) for i in range(3)]
    wq = torch.empty(G * N, K, dtype=torch.uint8, device=DEV)
    sw = torch.empty(G * N, dtype=torch.float32, device=DEV)
    for g in range(G):
        q, s = B.loka_quantize(synth.weight(K, N, seed=400 + g).to(DEV), B.SCALE_COL, transpose_out=True)
        wq[g * N:(g + 1) * N] = q
        sw[g * N:(g + 1) * N] = s
    # the library's choice for the shape, except where the case names a kernel that is not that choice
    variant = B.variant_id("panel32_256x256") if what.startswith("panel-synchronous kernel, FP8") else -1
    desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, norm, 1e-5, variant)

    x_in = torch.empty(rows, K, dtype=torch.bfloat16, device=DEV)
    xq = torch.empty(rows, K, dtype=torch.uint8, device=DEV)
    sx = torch.empty(rows, dtype=torch.float32, device=DEV)
    fp8 = "FP8 output" in what
    one_launch = "one launch" in what
    gamma, beta = (t.to(DEV) for t in synth.affine(N, seed=9)) if "gamma" in what else (None, None)
    gp, bp = (gamma.data_ptr(), beta.data_ptr()) if gamma is not None else (None, None)
    out = torch.empty(rows, N, dtype=torch.uint8 if fp8 else torch.bfloat16, device=DEV)
    so = torch.empty(rows, dtype=torch.float32, device=DEV)
    query = L.loka_fp8_gemm_norm_fp8out_workspace if fp8 else L.loka_fp8_gemm_norm_workspace
    ws_q = torch.empty(max(16, L.loka_quantize_workspace(B.SCALE_ROW, rows, K, 0)), dtype=torch.uint8, device=DEV)
    ws_g = torch.empty(max(16, query(ctypes.byref(desc))), dtype=torch.uint8, device=DEV)

    def step(stream):
        sp = ctypes.c_void_p(stream.cuda_stream)
        if one_launch:
            r = L.loka_fp8_linear_norm_xq(ctypes.byref(desc), x_in.data_ptr(), xq.data_ptr(), sx.data_ptr(), wq.data_ptr(),
                                          sw.data_ptr(), gp, bp, out.data_ptr(), None, sp)
            assert r == 0, r
            return
        r = L.loka_quantize(x_in.data_ptr(), rows, K, K, B.SCALE_ROW, 0, xq.data_ptr(), sx.data_ptr(), ws_q.data_ptr(),
                            ws_q.numel(), sp)
        assert r == 0, r
        if fp8:
            r = L.loka_fp8_gemm_norm_fp8out(ctypes.byref(desc), xq.data_ptr(), sx.data_ptr(), wq.data_ptr(), sw.data_ptr(), gp,
                                            bp, out.data_ptr(), so.data_ptr(), None, ws_g.data_ptr(), ws_g.numel(), sp)
        else:
            r = L.loka_fp8_gemm_norm(ctypes.byref(desc), xq.data_ptr(), sx.data_ptr(), wq.data_ptr(), sw.data_ptr(), gp,
                                     bp, out.data_ptr(), None, ws_g.data_ptr(), ws_g.numel(), sp)
        assert r == 0, r

    if one_launch:
        # the expected bits are those of the two eager calls
        desc.variant = B.variant_id("wreg32")
    # eager results for every input (also the warm-up that loads the code objects before the capture)
    cur = torch.cuda.current_stream()
    want = []
    for x in xs:
        x_in.copy_(x)
        step(cur)
        torch.cuda.synchronize()
        want.append((xq.clone(), sx.clone(), out.clone(), so.clone()))
        if one_launch:
            xq2, sx2 = B.loka_quantize(x, B.SCALE_ROW)
            o2, _ = B.loka_fp8_gemm_norm(desc, xq2, sx2, wq, sw, gamma, beta)
            torch.cuda.synchronize()
            assert torch.equal(xq, xq2) and torch.equal(sx, sx2) and torch.equal(out.view(torch.int16), o2.view(torch.int16))

    side = torch.cuda.Stream()
    side.wait_stream(cur)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    torch.cuda.synchronize()

    junk = torch.empty(1 << 20, device=DEV)
    for rep in range(6):
        i = rep % len(xs)
        x_in.copy_(xs[i])
        out.fill_(0)                    # eager work between the replays; stale results would show
        so.fill_(0)
        xq.fill_(0)
        junk.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xq, want[i][0]), f"{what}: codes, replay {rep}"
        assert torch.equal(sx, want[i][1]), f"{what}: scales, replay {rep}"
        assert torch.equal(out.view(torch.uint8), want[i][2].view(torch.uint8)), f"{what}: O, replay {rep}"
        if fp8:
            assert torch.equal(so, want[i][3]), f"{what}: output row scales, replay {rep}"
        if "panel" in what:
            assert B.loka_fp8_gemm_norm_check(desc, ws_g) == B.LOKA_OK
