"""The allocation-free entry point, loka_fp8_gemm_norm_static, against loka_fp8_gemm_norm (same kernels, the scratch
comes from the library's own device array): identical bits, on two calls in a row, the second with a smaller input
that finds the first call's leftovers in the array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_10886_amd import binding as B
from paper_2605_10886_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _operands(M, K, N, seed):
    x, w = synth.student_t4(M, K, seed=seed).to(DEV), synth.weight(K, N, seed=seed + 1).to(DEV)
    xq, sx = B.loka_quantize(x, B.SCALE_ROW)
    wq, sw = B.loka_quantize(w, B.SCALE_COL, transpose_out=True)
    return xq, sx, wq, sw


def test_static_scratch_gives_the_bits_of_the_workspace_call():
    L = B.lib()
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    gamma, beta = (t.to(DEV) for t in synth.affine(2048, seed=3))
    # rows wider than a tile: the panel kernel exchanges row statistics through the scratch.  First a larger problem,
    # then a smaller one with another tile count per row, then the first again.
    cases = [(2048, 256, 2048, "layernorm", True), (700, 384, 1280, "rmsnorm", False), (2048, 256, 2048, "layernorm", True)]
    for M, K, N, norm, affine in cases:
        xq, sx, wq, sw = _operands(M, K, N, seed=M + N)
        desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORMS[norm], 1e-5, variant=B.variant_id("panel32_256x256"))
        need = L.loka_fp8_gemm_norm_workspace(ctypes.byref(desc))
        assert 0 < need <= B.STATIC_SCRATCH_BYTES
        g = gamma[:N].contiguous() if affine else None
        b = beta[:N].contiguous() if affine else None
        ref, y_ref = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw, g, b, want_y=True)
        # outputs allocated before the call; the call itself gets plain pointers and allocates nothing
        out = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
        y = torch.empty(M, N, dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        st = L.loka_fp8_gemm_norm_static(ctypes.byref(desc), xq.data_ptr(), sx.data_ptr(), wq.data_ptr(), sw.data_ptr(),
                                         None if g is None else g.data_ptr(), None if b is None else b.data_ptr(),
                                         out.data_ptr(), y.data_ptr(), sp)
        assert st == B.LOKA_OK
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)) and torch.equal(y, y_ref)
        assert not bool(torch.isnan(out.float()).any())
    # the library's own choice of kernel, a shape without scratch, and a grouped launch
    for M, K, N, G in ((256, 128, 128, 1), (4096, 256, 256, 4)):
        xq, sx, wq, sw = _operands(G * M, K, N, seed=7)
        desc = B.make_desc(M, N, K, G, B.SCALE_ROW, B.SCALE_COL, B.NORM_RMSNORM, shared_w=True)
        ref, _ = B.loka_fp8_gemm_norm(desc, xq, sx, wq, sw)
        out, _ = B.loka_fp8_gemm_norm_static(desc, xq, sx, wq, sw)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16))


def test_static_scratch_rejects_what_does_not_fit():
    # the two-pass schedule stages fp32 Y in its workspace: far beyond the array at this size
    M, K, N = 8192, 256, 2048
    desc = B.make_desc(M, N, K, 1, B.SCALE_ROW, B.SCALE_COL, B.NORM_LAYERNORM, variant=B.variant_id("twopass128x128"))
    assert B.lib().loka_fp8_gemm_norm_workspace(ctypes.byref(desc)) > B.STATIC_SCRATCH_BYTES
    z8 = lambda *s: torch.zeros(*s, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.LokaError) as e:
        B.loka_fp8_gemm_norm_static(desc, z8(M, K), torch.ones(M, device=DEV), z8(N, K), torch.ones(N, device=DEV))
    assert e.value.status == B.LOKA_ERR_WORKSPACE
