"""The allocation-free weight gradient (cnn_conv_bwd_weight_static) against cnn_conv_bwd_weight, through the C ABI:
two calls in a row on the built-in scratch array, the second on a smaller layer, each bit for bit equal to the
workspace-based entry point (same kernels, same summation order) and within the contraction tolerance of the
oracle; a layer beyond the array's size is refused before anything is launched."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_1602_06709_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu

CASES = [  # N, C, H, W, K, R, S, stride, pad -- the second is smaller than the first
    (8, 64, 56, 56, 128, 3, 3, 1, 1),      # ring-buffer kernel, several splits
    (2, 24, 28, 20, 40, 3, 3, 1, 1),       # ragged feature counts, fewer splits: reads a prefix of the same array
    (4, 3, 64, 64, 32, 3, 3, 1, 1),        # first-layer kernel
    (4, 64, 56, 56, 64, 1, 1, 1, 0),       # implicit-GEMM kernel with a split contraction
]


def test_static_scratch_weight_gradient_matches_the_workspace_one(cnn):
    torch.cuda.set_device(0)
    ctx = cnn.Context()
    ref_ctx = cnn.Context()
    d = lambda a: torch.from_numpy(a).cuda()
    for i, (N, Cc, H, W, K, R, S, st, pad) in enumerate(CASES):
        print(f"case {i}: {(N, Cc, H, W, K, R, S, st, pad)}", flush=True)
        Pq, Q = cnn.out_dim(H, R, st, pad), cnn.out_dim(W, S, st, pad)
        x = synth.randn(91, 2 * i, (N, Cc, H, W)); dy = synth.randn(91, 2 * i + 1, (N, K, Pq, Q))
        need = cnn.lib().cnn_workspace_bytes(cnn.OP_CONV_BWD_WEIGHT, N, Cc, H, W, K, R, S, st, pad)
        assert need <= cnn.STATIC_SCRATCH_BYTES
        xd, dyd = d(x), d(dy)
        out = torch.full((K, Cc, R, S), float("nan"), dtype=torch.float32, device="cuda")
        ref = cnn.cnn_conv_bwd_weight(ref_ctx, xd, dyd, R, S, st, pad)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        cnn.cnn_conv_bwd_weight_static(ctx, xd, dyd, R, S, st, pad, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert ctx._ws is None                                   # no workspace was ever attached to this context
        assert torch.equal(out, ref), f"case {i}: differs from cnn_conv_bwd_weight"
        P.check_contraction(f"dw static {i}", P.np_(out), *oracle.conv_bwd_weight(x, dy, R, S, st, pad, with_abs=True))
    # a layer whose partial sums do not fit the built-in array: refused, nothing launched, output untouched
    N, Cc, H, W, K = 2, 2048, 14, 14, 2048
    need = cnn.lib().cnn_workspace_bytes(cnn.OP_CONV_BWD_WEIGHT, N, Cc, H, W, K, 3, 3, 1, 1)
    assert need > cnn.STATIC_SCRATCH_BYTES
    xd = torch.zeros((N, Cc, H, W), device="cuda"); dyd = torch.zeros((N, K, H, W), device="cuda")
    out = torch.full((K, Cc, 3, 3), 7.0, device="cuda")
    st = cnn.lib().cnn_conv_bwd_weight_static(ctx.handle, N, Cc, H, W, K, 3, 3, 1, 1, C.c_void_p(xd.data_ptr()),
                                              C.c_void_p(dyd.data_ptr()), C.c_void_p(out.data_ptr()))
    assert st == -3
    assert b"built-in scratch" in cnn.lib().cnn_last_error(ctx.handle)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    ctx.close(); ref_ctx.close()
