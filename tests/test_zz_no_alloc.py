"""svdmlp_forward_static_scratch (the entry point for callers that cannot allocate: per-forward buffers in the library's
static device array) against svdmlp_forward on the same context and inputs, through the C ABI, and against the fp64
oracle.  Two calls in a row share the array, the second with a smaller input, so whatever the first call left behind
(tickets, partial tiles, a longer activation) must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2510_25977_amd import binding as B
from paper_2510_25977_amd import synth

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2


def relmax(y, ref):
    return float(np.max(np.abs(y - ref)) / np.max(np.abs(ref)))


def _raw_forward(fn, ctx, X, M, Y):
    st = fn(ctx, ctypes.c_void_p(X.data_ptr()), int(M), ctypes.c_void_p(Y.data_ptr()),
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == B.SVDMLP_OK, B.status_string(st)


@pytest.mark.parametrize("d,ffn,r,rd,M1,M2", [(512, 1408, 192, 256, 100, 7), (4096, 14336, 512, 512, 16, 3),
                                             (512, 1408, 192, 256, 32, 32)])
def test_static_scratch_forward_matches_workspace_forward_twice_in_a_row(d, ffn, r, rd, M1, M2):
    dev = torch.device("cuda:0")
    L = B.lib()
    assert B.svdmlp_static_scratch_bytes() == 16 << 20
    gi = synth.make_gated(M1, d, ffn, r, rd, stream=61)
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    mlp = B.SvdMlp(max_M=M1, **f)
    a = {k: synth.to_f64(v) for k, v in gi.factors().items()}
    X1 = gi.X.to(dev)
    X2 = (gi.X[:M2] * 0.5 + 0.25).to(torch.bfloat16).to(dev).contiguous()   # other values, fewer rows
    for X, M in ((X1, M1), (X2, M2)):
        Yw = torch.full((M, d), 3.0, dtype=torch.bfloat16, device=dev)
        Ys = torch.full((M, d), -3.0, dtype=torch.bfloat16, device=dev)
        _raw_forward(L.svdmlp_forward, mlp.ctx, X, M, Yw)
        _raw_forward(L.svdmlp_forward_static_scratch, mlp.ctx, X, M, Ys)
        torch.cuda.synchronize()
        assert mlp.last_path == 3
        # same kernels, same fixed-order reductions: bit for bit
        assert torch.equal(Yw, Ys), (M, float((Yw.float() - Ys.float()).abs().max()))
        ref = oracle.gated(synth.to_f64(X.cpu()), **a)
        err = relmax(Ys.cpu().to(torch.float64).numpy(), ref)
        assert err <= BF16_TOL, (M, err)
    mlp.close()


def test_static_scratch_forward_rejects_what_does_not_fit_or_does_not_stream():
    dev = torch.device("cuda:0")
    L = B.lib()
    # 128 rows at ffn = 27648, r = 1024: T + H + Td = 7.8 MB, beyond the 7.5 MiB the array has for them
    gi = synth.make_gated(8, 256, 27648, 128, 128, stream=62)
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    mlp = B.SvdMlp(max_M=200, **f)
    X = torch.zeros((200, 256), dtype=torch.bfloat16, device=dev)
    Y = torch.full((200, 256), 5.0, dtype=torch.bfloat16, device=dev)
    args = lambda M: (mlp.ctx, ctypes.c_void_p(X.data_ptr()), M, ctypes.c_void_p(Y.data_ptr()), ctypes.c_void_p(0))
    assert L.svdmlp_forward_static_scratch(*args(129)) == B.SVDMLP_UNSUPPORTED      # not the weight-streaming path
    assert L.svdmlp_forward_static_scratch(*args(201)) == B.SVDMLP_INVALID_ARGUMENT
    assert L.svdmlp_forward_static_scratch(*args(0)) == B.SVDMLP_OK
    assert L.svdmlp_forward_static_scratch(*args(32)) == B.SVDMLP_OK                # 32 rows fit (1.8 MB)
    assert L.svdmlp_forward_static_scratch(*args(128)) == B.SVDMLP_OK               # 128 rows: 7.2 MB, fits
    mlp.close()
    gi = synth.make_gated(8, 256, 30720, 128, 128, stream=63)
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    mlp = B.SvdMlp(max_M=128, **f)
    args = lambda M: (mlp.ctx, ctypes.c_void_p(X.data_ptr()), M, ctypes.c_void_p(Y.data_ptr()), ctypes.c_void_p(0))
    assert L.svdmlp_forward_static_scratch(*args(128)) == B.SVDMLP_SCRATCH_TOO_SMALL  # 128 x 30720 x 2 = 7.9 MB
    assert "static scratch" in B.status_string(B.SVDMLP_SCRATCH_TOO_SMALL)
    assert L.svdmlp_forward_static_scratch(*args(64)) == B.SVDMLP_OK
    torch.cuda.synchronize()
    mlp.close()
    # fp32 contexts and the single factored layer have no such variant
    li = synth.make_linear_gaussian(8, 256, 512, 128, stream=64)
    lin = B.SvdMlp(max_M=8, Ug=li.U.to(dev), Vg=li.V.to(dev), kind=B.SVDMLP_LINEAR)
    Xl = li.X.to(dev)
    Ol = torch.empty((8, 512), dtype=torch.bfloat16, device=dev)
    assert L.svdmlp_forward_static_scratch(lin.ctx, ctypes.c_void_p(Xl.data_ptr()), 8, ctypes.c_void_p(Ol.data_ptr()),
                                           ctypes.c_void_p(0)) == B.SVDMLP_UNSUPPORTED
    lin.close()
