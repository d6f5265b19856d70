"""GPU parity: every libcnn entry point against the CPU oracle on the same seeded inputs.

Bar: bit-exact for permutations, ReLU and max-pool; for contractions rel-L2 <= 1e-5 and
|diff| <= 1e-4 * sum|a*b| per element.  All calls go through the C ABI (ctypes binding).
"""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_1602_06709_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx(cnn):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = cnn.Context()
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------------ config 1 (and the plain fallback kernels)
@pytest.mark.parametrize("force_direct", [0, 1])
def test_config1_single_conv_layer(cnn, ctx, force_direct):
    wl = synth.workload(1)
    x = synth.make_input(wl); w = synth.make_weights(wl)[0]; dy = synth.make_upstream(wl)
    say("config1 force_direct", force_direct, x.shape, w.shape, dy.shape)
    ctx.set_option(cnn.OPT_FORCE_DIRECT, force_direct)
    try:
        y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), 1, 1)
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), 32, 32, 1, 1)
        dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), 3, 3, 1, 1)
        wt = dev(w).clone()
        cnn.cnn_sgd_update(ctx, wt.view(-1), dw.view(-1), None, 0.01, 0.0)
        torch.cuda.synchronize()
    finally:
        ctx.set_option(cnn.OPT_FORCE_DIRECT, 0)
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, 1, 1, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, 32, 32, 1, 1, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, 3, 3, 1, 1, with_abs=True))
    wo, _ = oracle.sgd_update(w, P.np_(dw), None, 0.01, 0.0)
    P.check_elementwise("sgd", P.np_(wt), wo, atol_scale=np.abs(w).ravel() + 0.01 * np.abs(P.np_(dw)).ravel())


# ------------------------------------------------------------------ every tiled conv geometry, ragged edges
CONV_CASES = [  # N, C, H, K, R, pad       (square images, stride 1)
    (2, 16, 112, 40, 3, 1),     # 112-wide, ragged K
    (1, 8, 112, 136, 3, 1),     # two K tiles, second ragged
    (3, 24, 56, 64, 3, 1),      # K <= 64 path in backpropagation when roles swap
    (2, 16, 56, 130, 3, 1),
    (3, 16, 28, 72, 3, 1),      # images processed in pairs, odd N
    (5, 32, 14, 48, 3, 1),      # whole-image tile with 28 padded lanes
    (3, 8, 12, 136, 3, 1),      # pairs of 12x12 images
    (2, 8, 28, 40, 5, 0),       # 5x5, 28 -> 24
    (3, 64, 56, 128, 3, 1),
    (2, 8, 32, 136, 3, 1),      # 32x32 images: 8-block tiles
    (3, 12, 20, 40, 3, 1),      # 20x20: several images per tile, ragged
    (2, 8, 40, 130, 3, 0),      # pad 0: 40 -> 38
    (1, 16, 64, 24, 3, 2),      # pad 2: 64 -> 66
    (2, 8, 17, 72, 5, 2),       # 5x5 'same' on an odd size
    (2, 64, 28, 128, 3, 1),     # whole tiles: fixed-geometry weight gradient (two images per step), sliced contraction
    (5, 64, 14, 128, 3, 1),     # ... four images per step, odd N; pixel tiles cross image boundaries
    (3, 64, 12, 128, 3, 1),     # ... 12x12
    (7, 8, 7, 40, 3, 1),        # 7x7 images: one pixel tile spans several images
    (3, 128, 10, 24, 3, 1),     # long contraction, few outputs: every unit sliced
    (3, 96, 28, 40, 5, 0),      # 5x5 with 96 input features: backpropagation in 32-feature tiles (four wave columns)
    (2, 32, 20, 96, 5, 2),      # ... and the forward pass with 96 output features
    (3, 32, 28, 64, 5, 0),      # 5x5, 28 -> 24, whole tiles: fixed-geometry weight gradient, odd N
    (2, 16, 20, 40, 7, 3),      # 7x7 'same'
    (3, 32, 14, 72, 7, 0),      # 7x7, 14 -> 8
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_three_passes_tiled_geometries(cnn, ctx, case):
    N, C, H, K, R, pad = case
    say("conv case", case)
    x = synth.randn(90, 1, (N, C, H, H)); w = synth.randn(90, 2, (K, C, R, R), 0.1)
    P_ = H + 2 * pad - R + 1
    dy = synth.randn(90, 3, (N, K, P_, P_))
    y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), 1, pad)
    dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, H, 1, pad)
    dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, R, 1, pad)
    torch.cuda.synchronize()
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, 1, pad, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, H, 1, pad, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, R, 1, pad, with_abs=True))


# (N, C, H, K): 3x3 / pad 1 layers whose grid is within one round and spreads better in equal runs of chunks than
# in equal slices of units (54, 112 and 56 units on 256 compute units); a run ends one unit and begins the next
RUNS_CASES = [(20, 256, 14, 384), (32, 128, 14, 512), (8, 256, 28, 256)]


@pytest.mark.parametrize("case", RUNS_CASES)
def test_conv_units_dealt_out_in_runs_of_chunks(cnn, ctx, case):
    N, C, H, K = case
    say("runs-of-chunks case", case)
    x = np.maximum(synth.randn(82, 1, (N, C, H, H)), 0).astype(np.float32)
    w = synth.randn(82, 2, (K, C, 3, 3), 0.1)
    dy = synth.randn(82, 3, (N, K, H, H))
    ctx.profile_reset(); ctx.profile(True)
    y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), 1, 1)
    dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, H, 1, 1)
    torch.cuda.synchronize(); ctx.profile(False)
    names = [e[0] for e in ctx.profile_entries()]
    assert sum(" runs" in n for n in names) == 2, names
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, 1, 1, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, H, 1, 1, with_abs=True))
    # every epilogue runs in the reduction pass then: bit for bit the unfused sequences
    a = cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), 1, 1)
    assert torch.equal(a, cnn.cnn_relu_fwd(ctx, y))
    ap, arg = cnn.cnn_conv_fwd_relu_pool(ctx, dev(x), dev(w), 1, 1)
    ap2, arg2 = cnn.cnn_maxpool2_fwd(ctx, a)
    assert torch.equal(ap, ap2) and torch.equal(arg, arg2)
    dz = cnn.cnn_conv_bwd_data_relu(ctx, dev(dy), dev(w), dev(x), 1, 1)
    assert torch.equal(dz, cnn.cnn_relu_bwd(ctx, dev(x), dx))
    xp, xarg = cnn.cnn_maxpool2_fwd(ctx, dev(np.maximum(synth.randn(82, 4, (N, C, 2 * H, 2 * H)), 0).astype(np.float32)))
    du = cnn.cnn_conv_bwd_data_unpool_relu(ctx, dev(dy), dev(w), xarg, xp, 1, 1)
    assert du is not None
    ref = cnn.cnn_maxpool2_bwd(ctx, cnn.cnn_relu_bwd(ctx, xp, cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, H, 1, 1)), xarg, 2 * H, 2 * H)
    torch.cuda.synchronize()
    assert torch.equal(du, ref)


# (N, C, H, W, K, R, S, stride, pad): images that are not square, through every kernel family
RECT_CASES = [(2, 16, 20, 36, 40, 3, 3, 1, 1), (3, 8, 30, 14, 72, 3, 3, 1, 1), (2, 32, 12, 56, 130, 3, 3, 1, 1),
              (2, 16, 24, 40, 48, 5, 5, 1, 2), (2, 16, 18, 26, 40, 7, 7, 1, 3), (2, 3, 40, 64, 64, 3, 3, 1, 1),
              (2, 3, 51, 75, 96, 11, 11, 4, 0), (2, 3, 50, 70, 64, 7, 7, 2, 3), (2, 64, 14, 28, 128, 3, 3, 1, 1),
              (2, 16, 21, 33, 40, 3, 3, 2, 1)]


@pytest.mark.parametrize("case", RECT_CASES)
def test_conv_three_passes_rectangular_images(cnn, ctx, case):
    N, C, H, W, K, R, S, stride, pad = case
    say("rectangular case", case)
    P_, Q_ = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    x = synth.randn(89, 1, (N, C, H, W)); w = synth.randn(89, 2, (K, C, R, S), 0.1); dy = synth.randn(89, 3, (N, K, P_, Q_))
    y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), stride, pad)
    dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, stride, pad)
    dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, S, stride, pad)
    torch.cuda.synchronize()
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, stride, pad, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, W, stride, pad, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, S, stride, pad, with_abs=True))
    if P_ % 2 == 0 and Q_ % 2 == 0:
        r = cnn.cnn_conv_fwd_relu_pool(ctx, dev(x), dev(w), stride, pad)
        if r is not None:
            a2, arg2 = cnn.cnn_maxpool2_fwd(ctx, cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), stride, pad))
            torch.cuda.synchronize()
            assert torch.equal(r[0], a2) and torch.equal(r[1], arg2)


@pytest.mark.parametrize("case", [(2, 3, 64, 64, 7, 2, 3), (3, 3, 37, 40, 7, 2, 0), (2, 3, 224, 96, 7, 2, 3), (2, 1, 30, 24, 7, 1, 3)])
def test_first_layer_7x7(cnn, ctx, case):
    # few input features under a 7x7 kernel, stride 2 (and 1): single-chunk tiled forward, small-C weight gradient
    N, C, H, K, R, stride, pad = case
    say("7x7 first-layer case", case)
    P_ = (H + 2 * pad - R) // stride + 1
    x = synth.randn(91, 1, (N, C, H, H)); w = synth.randn(91, 2, (K, C, R, R), 0.1); dy = synth.randn(91, 3, (N, K, P_, P_))
    y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), stride, pad)
    dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, R, stride, pad)
    dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, H, stride, pad)
    torch.cuda.synchronize()
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, stride, pad, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, R, stride, pad, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, H, stride, pad, with_abs=True))


@pytest.mark.parametrize("force_direct", [0, 1])
def test_conv_generic_shapes_fall_back_and_match(cnn, ctx, force_direct):
    # strides, rectangular images, 11x11/4 and 1x1: served by whichever kernel applies; with force_direct by the
    # plain one-thread-per-output kernels
    ctx.set_option(cnn.OPT_FORCE_DIRECT, force_direct)
    try:
        _generic_shapes(cnn, ctx)
    finally:
        ctx.set_option(cnn.OPT_FORCE_DIRECT, 0)


def _generic_shapes(cnn, ctx):
    for (N, C, H, W, K, R, S, st, pad) in [(2, 3, 39, 39, 8, 11, 11, 4, 0), (1, 5, 9, 13, 7, 3, 2, 2, 1),
                                           (2, 4, 6, 6, 4, 1, 1, 1, 0), (1, 3, 224, 224, 8, 3, 3, 1, 1),
                                           (2, 3, 224, 224, 64, 3, 3, 1, 1), (3, 3, 231, 231, 96, 11, 11, 4, 0),
                                           (2, 3, 30, 30, 40, 3, 3, 1, 1), (1, 3, 24, 36, 20, 3, 3, 1, 0),
                                           (2, 8, 24, 36, 40, 3, 3, 1, 1), (2, 16, 31, 45, 72, 3, 3, 2, 1),
                                           (1, 8, 50, 30, 136, 5, 5, 2, 2), (2, 8, 13, 300, 16, 3, 3, 1, 1)]:
        say("generic conv", (N, C, H, W, K, R, S, st, pad))
        x = synth.randn(91, 1, (N, C, H, W)); w = synth.randn(91, 2, (K, C, R, S))
        y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), st, pad)
        dy = synth.randn(91, 3, tuple(y.shape))
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, st, pad)
        dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, S, st, pad)
        torch.cuda.synchronize()
        P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, st, pad, with_abs=True))
        P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, W, st, pad, with_abs=True))
        P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, S, st, pad, with_abs=True))


# (N, C, H, W, K, R, S, stride, pad): what only the implicit GEMM serves on the matrix cores. 1x1 (plain and strided),
# 3x3 / 5x5 strided with many input features (backpropagation and weight gradient), rectangular and even-sized
# kernels, 9x9, stride 3 and 4 with padding, tiles ragged in every dimension, a contraction shorter than one chunk
IGEMM_CASES = [(2, 256, 28, 28, 512, 1, 1, 1, 0), (3, 64, 56, 56, 128, 3, 3, 2, 1), (2, 96, 27, 27, 40, 1, 1, 2, 0),
               (2, 32, 30, 22, 72, 1, 7, 1, 3), (2, 24, 22, 30, 136, 7, 1, 1, 0), (2, 16, 20, 20, 33, 9, 9, 1, 4),
               (3, 20, 17, 23, 70, 2, 2, 2, 0), (2, 40, 33, 31, 64, 4, 4, 4, 2), (1, 130, 19, 19, 200, 3, 3, 3, 1),
               (2, 128, 28, 28, 256, 5, 5, 2, 2), (1, 5, 6, 6, 3, 2, 3, 1, 1), (65, 8, 9, 9, 16, 3, 2, 2, 1),
               # stride-1 3x3 with a prime width: the ring-buffer weight gradient has no column tile for it
               (2, 32, 20, 37, 48, 3, 3, 1, 1), (1, 24, 12, 67, 40, 3, 3, 1, 1),
               # no padding: gathered without coordinate checks (ragged rows, columns and contraction; strides 1 and 3)
               (2, 8, 24, 24, 24, 9, 9, 1, 0), (2, 12, 19, 21, 40, 4, 4, 1, 0), (3, 70, 13, 17, 90, 1, 1, 1, 0),
               (2, 33, 20, 22, 65, 1, 1, 3, 0)]


@pytest.mark.parametrize("case", IGEMM_CASES)
def test_conv_implicit_gemm_shapes(cnn, ctx, case):
    # the three passes, the ReLU forms of forward and backpropagation (bit-identical to the unfused sequence), and the
    # weight gradient with the SGD step folded in (bit-identical to gradient + update)
    N, C, H, W, K, R, S, st, pad = case
    say("implicit GEMM case", case)
    x = np.maximum(synth.randn(84, 1, (N, C, H, W)), 0).astype(np.float32)
    w = synth.randn(84, 2, (K, C, R, S), 0.2)
    y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), st, pad)
    dy = synth.randn(84, 3, tuple(y.shape))
    dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, st, pad)
    dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, S, st, pad)
    a = cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), st, pad)
    dz = cnn.cnn_conv_bwd_data_relu(ctx, dev(dy), dev(w), dev(x), st, pad)
    w0 = synth.randn(84, 4, (K, C, R, S), 0.05); v0 = synth.randn(84, 5, (K, C, R, S), 0.5)
    w1, v1 = dev(w0), dev(v0)
    assert cnn.cnn_conv_bwd_weight_sgd(ctx, dev(x), dev(dy), w1, v1, st, pad, 0.02, 0.9) is not None
    w2, v2 = dev(w0), dev(v0)
    cnn.cnn_sgd_update(ctx, w2.view(-1), dw.view(-1), v2.view(-1), 0.02, 0.9)
    torch.cuda.synchronize()
    P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, st, pad, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, W, st, pad, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, S, st, pad, with_abs=True))
    assert torch.equal(a, cnn.cnn_relu_fwd(ctx, y))
    assert torch.equal(dz, cnn.cnn_relu_bwd(ctx, dev(x), dx))
    assert torch.equal(w1, w2) and torch.equal(v1, v2)


def test_conv_tensors_beyond_two_gib(cnn, ctx):
    # an input of 2^29 + elements (byte offsets past 2^31): element offsets inside the kernels are 32-bit, byte
    # offsets must not be; a 3x3 layer (small output) and a 1x1 layer whose output is as large as its input;
    # sampled outputs, the first and the last element always among them
    N, C, H, W = 1, 32, 4100, 4100
    say("large tensor: generating", (N, C, H, W))
    x = synth.randn(83, 1, (N, C, H, W))
    xd = dev(x)
    for (K, R, pad) in [(8, 3, 1), (32, 1, 0)]:
        say("large tensor case", (N, C, H, W, K, R, pad))
        w = synth.randn(83, 2, (K, C, R, R), 0.2)
        dy = synth.randn(83, 3, (N, K, H, W))
        dyd, wd = dev(dy), dev(w)
        y = cnn.cnn_conv_fwd(ctx, xd, wd, 1, pad)
        dx = cnn.cnn_conv_bwd_data(ctx, dyd, wd, H, W, 1, pad)
        dw = cnn.cnn_conv_bwd_weight(ctx, xd, dyd, R, R, 1, pad)
        torch.cuda.synchronize()
        say("  checking")
        idx = np.unique(np.concatenate([P.sample(83, 10, y.numel(), 20000), [0, y.numel() - 1]]))
        ref, sabs = oracle.conv_fwd_at(x, w, idx, 1, pad)
        P.check_contraction("y", P.np_(y).ravel()[idx], ref, sabs)
        idx = np.unique(np.concatenate([P.sample(83, 11, dx.numel(), 20000), [0, dx.numel() - 1]]))
        ref, sabs = oracle.conv_bwd_data_at(dy, w, H, W, idx, 1, pad)
        P.check_contraction("dx", P.np_(dx).ravel()[idx], ref, sabs)
        idx = P.sample(83, 12, dw.numel(), 48)
        ref, sabs = oracle.conv_bwd_weight_at(x, dy, R, R, idx, 1, pad)
        P.check_contraction("dw", P.np_(dw).ravel()[idx], ref, sabs)
        del y, dx, dw, dyd


def test_conv_degenerate_shapes(cnn, ctx):
    # images of one pixel / one row / smaller than the kernel's reach, a single feature on either side, padding
    # beyond the kernel (outputs that see only zeros), a ragged 513-feature layer, one image
    for (N, C, H, W, K, R, S, st, pad) in [(1, 4, 3, 3, 1, 3, 3, 1, 1), (1, 16, 1, 1, 32, 3, 3, 1, 1), (1, 4, 2, 50, 8, 3, 3, 1, 1),
                                           (1, 8, 5, 5, 40, 3, 3, 1, 3), (2, 16, 8, 8, 16, 5, 5, 1, 4), (2, 1, 8, 8, 1, 3, 3, 1, 1),
                                           (1, 4, 8, 8, 513, 3, 3, 1, 1), (1, 64, 14, 14, 128, 3, 3, 1, 1), (1, 3, 7, 7, 5, 7, 7, 2, 3),
                                           (3, 16, 4, 4, 8, 7, 7, 1, 3), (1, 3, 11, 11, 96, 11, 11, 4, 0)]:
        say("degenerate conv", (N, C, H, W, K, R, S, st, pad))
        x = synth.randn(88, 1, (N, C, H, W)); w = synth.randn(88, 2, (K, C, R, S))
        y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), st, pad)
        dy = synth.randn(88, 3, tuple(y.shape))
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, st, pad)
        dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, S, st, pad)
        torch.cuda.synchronize()
        P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, st, pad, with_abs=True))
        P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, W, st, pad, with_abs=True))
        P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, S, st, pad, with_abs=True))


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 3, 3, 3, 5, 5, 7]))
        st = int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.integers(0, R // 2 + 2))
        H, W = int(rng.integers(R, 44)), int(rng.integers(R, 44))
        C = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 32, 64, 96]))
        K = int(rng.choice([1, 8, 31, 32, 40, 64, 72, 96, 128, 136]))
        N = int(rng.integers(1, 6))
        if (H + 2 * pad - R) // st + 1 < 1 or (W + 2 * pad - R) // st + 1 < 1:
            continue
        out.append((N, C, H, W, K, R, R, st, pad))
    return out


@pytest.mark.parametrize("chunk", [0, 1, 2])
def test_conv_seeded_random_shapes(cnn, ctx, chunk):
    # 3 x 14 seeded shapes over kernel sizes 1 / 3 / 5 / 7, strides 1 / 2, paddings up to R/2 + 1, ragged feature
    # counts and rectangular images: whichever kernel serves each pass must match the oracle
    for case in _random_shapes(14, 1000 + chunk):
        N, C, H, W, K, R, S, st, pad = case
        say("random conv", case)
        x = synth.randn(86, 1, (N, C, H, W)); w = synth.randn(86, 2, (K, C, R, S), 0.2)
        y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), st, pad)
        dy = synth.randn(86, 3, tuple(y.shape))
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, st, pad)
        dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, S, st, pad)
        torch.cuda.synchronize()
        P.check_contraction("y", P.np_(y), *oracle.conv_fwd(x, w, st, pad, with_abs=True))
        P.check_contraction("dx", P.np_(dx), *oracle.conv_bwd_data(dy, w, H, W, st, pad, with_abs=True))
        P.check_contraction("dw", P.np_(dw), *oracle.conv_bwd_weight(x, dy, R, S, st, pad, with_abs=True))


def test_conv_seeded_random_large_layers(cnn, ctx):
    # 30 seeded layers with 64 ... 1024 features at 7 ... 56 pixels and minibatches up to 64 (several rounds of tiles, tail
    # slices, runs of chunks, split weight gradients), outputs sampled against the oracle
    rng = np.random.default_rng(2000)
    done = 0
    while done < 30:
        R = int(rng.choice([3, 3, 3, 5, 7])); pad = int(rng.choice([0, (R - 1) // 2]))
        H = int(rng.choice([7, 12, 14, 24, 28, 56, 30])); W = H if rng.random() < 0.7 else int(rng.choice([14, 28, 40]))
        C = int(rng.choice([64, 96, 128, 256, 512])); K = int(rng.choice([64, 128, 192, 256, 512, 1024]))
        N = int(rng.integers(1, 65))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        P_, Q_ = H + 2 * pad - R + 1, W + 2 * pad - R + 1
        while N > 1 and N * C * K * R * R * P_ * Q_ > 4e10:
            N //= 2
        say("random large layer", (N, C, H, W, K, R, pad))
        x = np.maximum(synth.randn(85, 3 * done, (N, C, H, W)), 0).astype(np.float32)
        w = synth.randn(85, 3 * done + 1, (K, C, R, R), 0.05); dy = synth.randn(85, 3 * done + 2, (N, K, P_, Q_))
        y = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), 1, pad)
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, W, 1, pad)
        dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, R, 1, pad)
        torch.cuda.synchronize()
        idx = P.sample(85, 1000 + done, y.numel(), 4000)
        P.check_contraction("y", P.np_(y).ravel()[idx], *oracle.conv_fwd_at(x, w, idx, 1, pad))
        idx = P.sample(85, 2000 + done, dx.numel(), 4000)
        P.check_contraction("dx", P.np_(dx).ravel()[idx], *oracle.conv_bwd_data_at(dy, w, H, W, idx, 1, pad))
        idx = P.sample(85, 3000 + done, dw.numel(), 300)
        P.check_contraction("dw", P.np_(dw).ravel()[idx], *oracle.conv_bwd_weight_at(x, dy, R, R, idx, 1, pad))
        done += 1


def test_bwd_weight_is_bitwise_repeatable(cnn, ctx):
    x = dev(synth.randn(92, 1, (4, 32, 28, 28))); dy = dev(synth.randn(92, 2, (4, 64, 28, 28)))
    a = cnn.cnn_conv_bwd_weight(ctx, x, dy, 3, 3, 1, 1).clone()
    b = cnn.cnn_conv_bwd_weight(ctx, x, dy, 3, 3, 1, 1)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ------------------------------------------------------------------ fully connected
FC_CASES = [(64, 1024, 1000), (64, 440, 2048), (5, 36, 20), (130, 256, 136), (256, 2048, 520), (64, 25088, 256),
            (1, 4096, 1024), (7, 100, 52), (33, 260, 1000), (1024, 64, 64), (300, 1028, 260), (4, 8, 4),
            # more tiles than resident workgroups with a short last round: the tail tiles are sliced along the
            # contraction (forward of the first, weight gradient of the second)
            (1024, 512, 9304), (512, 2304, 4104)]


@pytest.mark.parametrize("case", FC_CASES)
def test_fc_three_passes(cnn, ctx, case):
    N, I, O = case
    say("fc case", case)
    x = synth.randn(93, 1, (N, I)); w = synth.randn(93, 2, (O, I), 0.05); dy = synth.randn(93, 3, (N, O))
    y = cnn.cnn_fc_fwd(ctx, dev(x), dev(w))
    dx, dw = cnn.cnn_fc_bwd(ctx, dev(x), dev(w), dev(dy))
    dx_only, none = cnn.cnn_fc_bwd(ctx, None, dev(w), dev(dy), need_dw=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(dx_only, dx)
    P.check_contraction("y", P.np_(y), *oracle.fc_fwd(x, w, with_abs=True))
    P.check_contraction("dx", P.np_(dx), *oracle.fc_bwd_data(dy, w, with_abs=True))
    P.check_contraction("dw", P.np_(dw), *oracle.fc_bwd_weight(x, dy, with_abs=True))


@pytest.mark.parametrize("case", [(64, 1024, 1000), (130, 256, 136), (256, 2048, 520), (64, 25088, 256), (1024, 64, 64),
                                  (300, 1028, 260), (1024, 512, 9304), (1024, 2048, 2048), (4, 8, 4)])
def test_fc_with_the_activation_folded_into_the_store(cnn, ctx, case):
    # forward: act(x W^T); backward: the derivative of the activation that produced x folded into dx, with and without
    # the SGD step -- each bit for bit equal to the unfused sequence (one tile, split contraction, sliced tail tiles)
    N, I, O = case
    say("fc+act case", case)
    w0 = synth.randn(93, 2, (O, I), 0.05); dy = synth.randn(93, 3, (N, O)); v0 = synth.randn(93, 4, (O, I), 0.5)
    z_in = synth.randn(93, 1, (N, I))
    for act in ("relu", "sigmoid"):
        x = P.np_(cnn.cnn_relu_fwd(ctx, dev(z_in)) if act == "relu" else cnn.cnn_sigmoid_fwd(ctx, dev(z_in)))   # an activation's output
        a = cnn.cnn_fc_fwd_act(ctx, dev(x), dev(w0), act)
        assert a is not None
        z = cnn.cnn_fc_fwd(ctx, dev(x), dev(w0))
        ref_a = cnn.cnn_relu_fwd(ctx, z) if act == "relu" else cnn.cnn_sigmoid_fwd(ctx, z)
        assert torch.equal(a, ref_a), f"{act}: folded forward differs from fc_fwd + activation"
        dz, dw = cnn.cnn_fc_bwd_act(ctx, dev(x), dev(w0), dev(dy), act)
        dx_u, dw_u = cnn.cnn_fc_bwd(ctx, dev(x), dev(w0), dev(dy))
        ref_dz = cnn.cnn_relu_bwd(ctx, dev(x), dx_u) if act == "relu" else cnn.cnn_sigmoid_bwd(ctx, dev(x), dx_u)
        assert torch.equal(dz, ref_dz) and torch.equal(dw, dw_u), f"{act}: folded backward differs from the unfused sequence"
        w, v = dev(w0), dev(v0)
        r = cnn.cnn_fc_bwd_sgd_act(ctx, dev(x), w, dev(dy), act, v, None, 0.01, 0.9)
        w2, v2 = dev(w0), dev(v0)
        r2 = cnn.cnn_fc_bwd_sgd(ctx, dev(x), w2, dev(dy), v2, True, None, 0.01, 0.9)
        torch.cuda.synchronize()
        assert r is not None and torch.equal(r[0], ref_dz) and torch.equal(w, w2) and torch.equal(v, v2)
        # against the oracle
        lay = [("fc", I, O)]
        P.check_trace_item(("fc_fwd_act", 0, 0, dev(x), dev(w0), a, act), 93, lay, True)
        P.check_trace_item(("fc_bwd_act", 0, 0, dev(x), dev(w0), dev(dy), dz, dw, act), 93, lay, True)
    # shapes only the plain kernels serve are refused, nothing written
    xo = dev(synth.randn(93, 5, (5, 6))); wo = dev(synth.randn(93, 6, (10, 6))); out = torch.full((5, 10), 7.0, device="cuda")
    assert cnn.cnn_fc_fwd_act(ctx, xo, wo, "relu", out=out) is None
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


# ------------------------------------------------------------------ SGD, layouts, glue
@pytest.mark.parametrize("n", [1, 3, 4, 1027, 1 << 20, (1 << 22) + 5])
def test_sgd_update(cnn, ctx, n):
    w = synth.randn(94, 1, (n,)); g = synth.randn(94, 2, (n,)); v = synth.randn(94, 3, (n,))
    wt, vt = dev(w), dev(v)
    cnn.cnn_sgd_update(ctx, wt, dev(g), vt, 0.01, 0.9)
    w2 = dev(w)
    cnn.cnn_sgd_update(ctx, w2, dev(g), None, 0.01, 0.0)
    torch.cuda.synchronize()
    wo, vo = oracle.sgd_update(w, g, v, 0.01, 0.9)
    P.check_elementwise("v", P.np_(vt), vo, atol_scale=np.abs(v) + np.abs(g))
    P.check_elementwise("w", P.np_(wt), wo, atol_scale=np.abs(w) + 0.01 * (np.abs(v) + np.abs(g)))
    wo, _ = oracle.sgd_update(w, g, None, 0.01, 0.0)
    P.check_elementwise("w0", P.np_(w2), wo, atol_scale=np.abs(w) + 0.01 * np.abs(g))


def test_measurement_probes(cnn, ctx):
    # the stream probes move what they say they move; the MFMA probe reports its FLOPs and leaves finite numbers
    for n in (4, 2048 + 4, (1 << 20) + 12):
        src = torch.arange(n, dtype=torch.float32, device="cuda"); dst = torch.full((n + 4,), -1.0, device="cuda")
        cnn.cnn_probe_stream(ctx, cnn.STREAM_COPY, src, dst[:n])
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and bool((dst[n:] == -1.0).all())
        cnn.cnn_probe_stream(ctx, cnn.STREAM_WRITE, None, dst[:n])
        cnn.cnn_probe_stream(ctx, cnn.STREAM_READ, src, dst[:n])
        torch.cuda.synchronize()
        assert torch.equal(dst[:n].view(-1, 4), torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").expand(n // 4, 4))
        assert bool((dst[n:] == -1.0).all())
    sink = torch.zeros(cnn.PROBE_SINK_FLOATS, device="cuda")
    fl = cnn.cnn_probe_mfma(ctx, 10, sink)
    torch.cuda.synchronize()
    assert fl == 512 * 4 * 10 * 8 * 4096.0 and bool(torch.isfinite(sink).all()) and float(sink.abs().sum()) > 0
    assert cnn.lib().cnn_probe_stream(ctx.handle, 3, 8, src.data_ptr(), dst.data_ptr()) == -1
    assert cnn.lib().cnn_probe_stream(ctx.handle, 2, 6, src.data_ptr(), dst.data_ptr()) == -1


# (N, C, H, K, R, stride, pad): whole-tile and ragged 3x3, 5x5, the two first-layer kernels, one split / many splits
WSGD_CASES = [(4, 64, 28, 128, 3, 1, 1), (3, 16, 28, 72, 3, 1, 1), (2, 32, 12, 64, 5, 1, 2), (2, 3, 32, 64, 3, 1, 1),
              (2, 3, 63, 96, 11, 4, 0), (8, 128, 14, 256, 3, 1, 1), (1, 64, 56, 128, 3, 1, 1)]


@pytest.mark.parametrize("case", WSGD_CASES)
def test_conv_weight_gradient_with_the_sgd_step_folded_in(cnn, ctx, case):
    N, C, H, K, R, stride, pad = case
    say("wgrad+sgd case", case)
    P_ = (H + 2 * pad - R) // stride + 1
    x = synth.randn(95, 1, (N, C, H, H)); dy = synth.randn(95, 2, (N, K, P_, P_))
    w0 = synth.randn(95, 3, (K, C, R, R), 0.05); v0 = synth.randn(95, 4, (K, C, R, R), 0.5)
    g_ref, sabs = oracle.conv_bwd_weight(x, dy, R, R, stride, pad, with_abs=True)
    dw = cnn.cnn_conv_bwd_weight(ctx, dev(x), dev(dy), R, R, stride, pad)
    for lr, mu, use_v in [(0.01, 0.9, True), (0.05, 0.0, False)]:
        w, v = dev(w0), (dev(v0) if use_v else None)
        assert cnn.cnn_conv_bwd_weight_sgd(ctx, dev(x), dev(dy), w, v, stride, pad, lr, mu) is not None
        w2, v2 = dev(w0), (dev(v0) if use_v else None)
        cnn.cnn_sgd_update(ctx, w2.view(-1), dw.view(-1), v2.view(-1) if use_v else None, lr, mu)
        torch.cuda.synchronize()
        assert torch.equal(w, w2), "folded update differs from gradient + cnn_sgd_update"
        if use_v:
            assert torch.equal(v, v2)
        P.check_fused_update(f"wsgd{case}", w0, v0 if use_v else None, g_ref, sabs, w, v, lr, mu)


def _mirrored_transpose(w):
    """wT[c][k][r][s] = w[k][c][R-1-r][S-1-s], by torch indexing (a permutation: exact)."""
    return w.flip(2, 3).transpose(0, 1).contiguous()


@pytest.mark.parametrize("case", [(4, 64, 28, 128, 3, 1, 1), (3, 16, 28, 72, 3, 1, 1), (2, 32, 12, 64, 5, 1, 2), (2, 24, 14, 40, 7, 1, 3),
                                  (8, 128, 14, 256, 3, 1, 1), (2, 32, 20, 48, 1, 1, 0), (2, 16, 15, 24, 3, 2, 1)])
def test_resident_transpose_weights(cnn, ctx, case):
    # Section 2.3's transpose-weights kept beside the weights: made once, read by the three backpropagation forms
    # (same bits as the calls that transpose per call), refreshed by the folded update (ring-buffer kernel: inside the
    # reduction; other kernels: by a transpose behind the update)
    N, C, H, K, R, stride, pad = case
    say("resident wT case", case)
    P_ = (H + 2 * pad - R) // stride + 1
    w0 = synth.randn(92, 1, (K, C, R, R), 0.05); v0 = synth.randn(92, 2, (K, C, R, R), 0.5)
    x = np.maximum(synth.randn(92, 3, (N, C, H, H)), 0).astype(np.float32); dy = synth.randn(92, 4, (N, K, P_, P_))
    w = dev(w0)
    wT = cnn.cnn_conv_transpose_weights(ctx, w)
    assert wT is not None and torch.equal(wT, _mirrored_transpose(w))
    served = cnn.cnn_conv_bwd_data_wt(ctx, dev(dy), wT, H, H, stride, pad)
    if stride != 1 or R == 1:
        assert served is None                       # only the implicit GEMM serves these: the plain calls remain
    else:
        assert torch.equal(served, cnn.cnn_conv_bwd_data(ctx, dev(dy), w, H, H, stride, pad))
        assert torch.equal(cnn.cnn_conv_bwd_data_wt(ctx, dev(dy), wT, H, H, stride, pad, x_act=dev(x)),
                           cnn.cnn_conv_bwd_data_relu(ctx, dev(dy), w, dev(x), stride, pad))
        arg = torch.from_numpy(synth.rng(92, 5).integers(0, 4, (N, C, H, H)).astype(np.uint8)).cuda()
        ref = cnn.cnn_conv_bwd_data_unpool_relu(ctx, dev(dy), w, arg, dev(x), stride, pad)
        got = cnn.cnn_conv_bwd_data_wt(ctx, dev(dy), wT, H, H, stride, pad, x_act=dev(x), arg=arg)
        assert (ref is None and got is None) or torch.equal(got, ref)
    # two folded updates in a row: the second one starts from the first one's weights and velocity
    w1, v1, w2, v2 = dev(w0), dev(v0), dev(w0), dev(v0)
    for it in range(2):
        assert cnn.cnn_conv_bwd_weight_sgd_wt(ctx, dev(x), dev(dy), w1, wT, v1, stride, pad, 0.01, 0.9) is not None
        assert cnn.cnn_conv_bwd_weight_sgd(ctx, dev(x), dev(dy), w2, v2, stride, pad, 0.01, 0.9) is not None
        torch.cuda.synchronize()
        assert torch.equal(w1, w2) and torch.equal(v1, v2), f"update {it}: weights differ from cnn_conv_bwd_weight_sgd"
        assert torch.equal(wT, _mirrored_transpose(w1)), f"update {it}: transpose-weights not current"


def test_training_steps_keep_the_resident_transpose_weights_current(cnn, ctx):
    # VGG-A's convolution stack at minibatch 4 with an update: after every step each convolution's transpose-weights
    # equal the mirrored transpose of its weights; same weights as a net that transposes per call
    from paper_1602_06709_amd.net import Net
    wl = dataclasses.replace(synth.workload(2), sgd=True, lr=1e-5, momentum=0.9)    # small steps: everything stays finite
    nets = [Net(ctx, wl, synth.make_weights(wl), resident_wt=r) for r in (True, False)]
    for it in range(3):
        for net in nets:
            net.set_input(synth.make_input(wl)); net.set_upstream(synth.make_upstream(wl))
            net.step()
        torch.cuda.synchronize()
        assert bool(torch.isfinite(nets[0].w_arena).all())
        assert torch.equal(nets[0].w_arena, nets[1].w_arena) and torch.equal(nets[0].v_arena, nets[1].v_arena)
        kept = [wi for wi, t in enumerate(nets[0].wT) if t is not None]
        assert len(kept) == 7 and all(nets[0]._wt_state[wi] == "fresh" for wi in kept)
        for wi in kept:
            assert torch.equal(nets[0].wT[wi], _mirrored_transpose(nets[0].w[wi])), f"step {it} layer {wi}"
    assert all(t is None for t in nets[1].wT)


def test_folded_sgd_refuses_what_only_the_plain_kernels_serve(cnn, ctx):
    x = dev(synth.randn(95, 5, (2, 5, 9, 9))); dy = dev(synth.randn(95, 6, (2, 7, 9, 9)))
    w0 = synth.randn(95, 7, (7, 5, 3, 3)); w = dev(w0)
    ctx.set_option(cnn.OPT_FORCE_DIRECT, 1)
    try:
        assert cnn.cnn_conv_bwd_weight_sgd(ctx, x, dy, w, None, 1, 1, 0.1, 0.0) is None
    finally:
        ctx.set_option(cnn.OPT_FORCE_DIRECT, 0)
    xf = dev(synth.randn(95, 8, (5, 6))); dyf = dev(synth.randn(95, 9, (5, 10)))     # I % 4 != 0
    wf0 = synth.randn(95, 10, (10, 6)); wf = dev(wf0)
    dxf = torch.full((5, 6), 7.0, device="cuda")
    assert cnn.cnn_fc_bwd_sgd(ctx, xf, wf, dyf, None, True, dxf, 0.1, 0.0) is None
    torch.cuda.synchronize()
    assert np.array_equal(P.np_(w), w0) and np.array_equal(P.np_(wf), wf0) and bool((dxf == 7.0).all())


@pytest.mark.parametrize("case", FC_CASES + [(64, 25088, 512)])
def test_fc_backward_with_the_sgd_step_folded_in(cnn, ctx, case):
    N, I, O = case
    if I % 4 or O % 4:
        pytest.skip("served by the plain kernels only (covered by the refusal test)")
    say("fc+sgd case", case)
    x = synth.randn(96, 1, (N, I)); w0 = synth.randn(96, 2, (O, I), 0.05); dy = synth.randn(96, 3, (N, O))
    v0 = synth.randn(96, 4, (O, I), 0.5)
    g_ref, sabs = oracle.fc_bwd_weight(x, dy, with_abs=True)
    dx_u, dw = cnn.cnn_fc_bwd(ctx, dev(x), dev(w0), dev(dy))
    for lr, mu, use_v in [(0.01, 0.9, True), (0.05, 0.0, False)]:
        w, v = dev(w0), (dev(v0) if use_v else None)
        r = cnn.cnn_fc_bwd_sgd(ctx, dev(x), w, dev(dy), v, True, None, lr, mu)
        assert r is not None
        w2, v2 = dev(w0), (dev(v0) if use_v else None)
        cnn.cnn_sgd_update(ctx, w2.view(-1), dw.view(-1), v2.view(-1) if use_v else None, lr, mu)
        torch.cuda.synchronize()
        assert torch.equal(r[0], dx_u), "dx must come from the weights before the update"
        assert torch.equal(w, w2) and (not use_v or torch.equal(v, v2))
        P.check_fused_update(f"fcsgd{case}", w0, v0 if use_v else None, g_ref, sabs, w, v, lr, mu)
    # first layer: no dx
    w = dev(w0)
    r = cnn.cnn_fc_bwd_sgd(ctx, dev(x), w, dev(dy), None, False, None, 0.05, 0.0)
    torch.cuda.synchronize()
    assert r is not None and r[0] is None and torch.equal(w, w2)


@pytest.mark.parametrize("sw", [4, 8, 16, 32])
def test_blocked_layouts_bit_exact(cnn, ctx, sw):
    x = synth.randn(95, 1, (3, 19, 7, 5)); w = synth.randn(95, 2, (21, 19, 3, 3))
    xp = cnn.cnn_pack_act(ctx, dev(x), sw)
    assert np.array_equal(P.np_(xp), oracle.pack_act(x, sw))
    assert np.array_equal(P.np_(cnn.cnn_unpack_act(ctx, xp, 19)), x)
    for tr in (False, True):
        wp = cnn.cnn_pack_wt(ctx, dev(w), sw, tr)
        assert np.array_equal(P.np_(wp), oracle.pack_wt(w, sw, tr))
        assert np.array_equal(P.np_(cnn.cnn_unpack_wt(ctx, wp, 21, 19, tr)), w)


def test_glue_ops(cnn, ctx):
    z = synth.randn(96, 1, (3, 5, 8, 12)); z[0, 0, 0, :4] = 0.0; da = synth.randn(96, 2, z.shape)
    assert np.array_equal(P.np_(cnn.cnn_relu_fwd(ctx, dev(z))).astype(np.float64), oracle.relu_fwd(z))
    assert np.array_equal(P.np_(cnn.cnn_relu_bwd(ctx, dev(z), dev(da))).astype(np.float64), oracle.relu_bwd(z, da))
    zt = z.copy(); zt[1, 2, 2:4, 4:6] = 7.0          # a tie inside one window
    y, arg = cnn.cnn_maxpool2_fwd(ctx, dev(zt))
    yo, ao = oracle.maxpool2_fwd(zt)
    assert np.array_equal(P.np_(y).astype(np.float64), yo) and np.array_equal(P.np_(arg).astype(np.int32), ao)
    dy = synth.randn(96, 3, tuple(y.shape))
    assert np.array_equal(P.np_(cnn.cnn_maxpool2_bwd(ctx, dev(dy), arg, 8, 12)).astype(np.float64),
                          oracle.maxpool2_bwd(dy, ao, 8, 12))
    a = cnn.cnn_sigmoid_fwd(ctx, dev(z))
    P.check_elementwise("sigmoid", P.np_(a), oracle.sigmoid_fwd(z), ulps=8)
    P.check_elementwise("sigmoid_bwd", P.np_(cnn.cnn_sigmoid_bwd(ctx, a, dev(da))), oracle.sigmoid_bwd(P.np_(a), da),
                        atol_scale=np.abs(da) * 0.25)
    # 1000 and 9304 classes: the row stays in LDS; 12007: three passes over memory; 3: fewer classes than threads
    for O in (1000, 9304, 12007, 3):
        lg = synth.randn(96, 4, (7, O), 3.0); lab = synth.rng(96, 5).integers(0, O, 7).astype(np.int32)
        loss, dz = cnn.cnn_softmax_xent(ctx, dev(lg), torch.from_numpy(lab).cuda())
        lo, dzo = oracle.softmax_xent(lg, lab)
        assert abs(float(P.np_(loss).astype(np.float64).mean()) - lo) < 1e-5 * abs(lo)
        assert np.linalg.norm(P.np_(dz) - dzo) / np.linalg.norm(dzo) < 1e-5
    # a label outside [0, O): NaN loss for that sample only, nothing read out of bounds, no -1 term in its row
    bad = lab.copy(); bad[2] = O + 5
    loss, dz = cnn.cnn_softmax_xent(ctx, dev(lg), torch.from_numpy(bad).cuda())
    ln = P.np_(loss)
    assert np.isnan(ln[2]) and np.all(np.isfinite(np.delete(ln, 2))) and np.all(P.np_(dz)[2] >= 0)


def test_argument_validation_launches_nothing(cnn, ctx):
    L = cnn.lib(); h = ctx.handle
    x = dev(np.zeros((1, 1, 4, 4), np.float32))
    assert L.cnn_conv_fwd(h, 1, 1, 4, 4, 1, 3, 3, 0, 1, x.data_ptr(), x.data_ptr(), x.data_ptr()) == -1   # stride 0
    assert L.cnn_conv_fwd(h, 1, 1, 2, 2, 1, 5, 5, 1, 0, x.data_ptr(), x.data_ptr(), x.data_ptr()) == -1   # empty output
    assert L.cnn_conv_fwd(h, 1, 1, 4, 4, 1, 3, 3, 1, 1, None, x.data_ptr(), x.data_ptr()) == -1
    assert L.cnn_conv_fwd(h, 1, 1, 4, 4, 1, 3, 3, 1, 1, x.data_ptr() + 4, x.data_ptr(), x.data_ptr()) == -1
    assert L.cnn_sgd_update(h, 0, x.data_ptr(), x.data_ptr(), None, 0.1, 0.0) == -1


# ------------------------------------------------------------------ the network workloads, per call, teacher-forced
def _run_and_check(cnn, ctx, cfg, N, full, fuse=True, fuse_pool=True, **kw):
    from paper_1602_06709_amd.net import Net
    wl = synth.workload(cfg, N)
    say(f"workload cfg{cfg} N={wl.input_shape[0]} full={full} fuse={fuse} fuse_pool={fuse_pool}")
    net = Net(ctx, wl, synth.make_weights(wl), record=True, fuse=fuse, fuse_pool=fuse_pool)
    net.set_input(synth.make_input(wl), synth.make_labels(wl) if wl.loss else None)
    net.forward()
    if wl.loss:
        net.loss()
    else:
        net.set_upstream(synth.make_upstream(wl))
    net.backward()
    torch.cuda.synchronize()
    worst = 0.0
    for item in net.trace:
        r = P.check_trace_item(item, cfg, wl.layers, full, **kw)
        say(f"  {item[0]}@{item[1]} rel-L2 {r:.2e}")
        worst = max(worst, r)
    if wl.sgd:
        w0 = P.np_(net.w_arena).copy(); g = P.np_(net.dw_arena).copy()
        v0 = P.np_(net.v_arena).copy() if net.v_arena is not None else None
        net.sgd(); torch.cuda.synchronize()
        wo, vo = oracle.sgd_update(w0, g, v0, wl.lr, wl.momentum)
        P.check_elementwise("sgd:w", P.np_(net.w_arena), wo,
                            atol_scale=np.abs(w0) + wl.lr * (np.abs(g) + (np.abs(v0) if v0 is not None else 0)))
        if vo is not None:
            P.check_elementwise("sgd:v", P.np_(net.v_arena), vo, atol_scale=np.abs(v0) + np.abs(g))
    return worst


@pytest.mark.parametrize("fuse", [True, "no-pool", False])
def test_config2_vgg_a_conv_stack_n4_full_tensors(cnn, ctx, fuse):
    _run_and_check(cnn, ctx, 2, None, True, fuse=bool(fuse), fuse_pool=fuse is True)


def test_fused_relu_entry_points_equal_the_unfused_sequence(cnn, ctx):
    # conv_fwd_relu == relu(conv_fwd); conv_bwd_data_relu == relu_bwd(x, conv_bwd_data); pool_relu_bwd == relu_bwd(pool_bwd)
    # (the 64- and 128-channel cases slice the contraction, so the epilogue runs in the tile reduction)
    for (N, C, H, K, R, pad) in [(3, 16, 28, 72, 3, 1), (2, 3, 224, 64, 3, 1), (5, 32, 14, 48, 3, 1), (2, 8, 28, 40, 5, 0),
                                 (2, 5, 9, 7, 3, 1), (2, 64, 28, 128, 3, 1), (3, 128, 10, 64, 3, 1)]:
        say("fused case", (N, C, H, K, R, pad))
        x = np.maximum(synth.randn(97, 1, (N, C, H, H)), 0).astype(np.float32)      # a ReLU output
        w = synth.randn(97, 2, (K, C, R, R), 0.1)
        P_ = H + 2 * pad - R + 1
        dy = synth.randn(97, 3, (N, K, P_, P_))
        a = cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), 1, pad)
        z = cnn.cnn_conv_fwd(ctx, dev(x), dev(w), 1, pad)
        assert torch.equal(a, cnn.cnn_relu_fwd(ctx, z))
        dz = cnn.cnn_conv_bwd_data_relu(ctx, dev(dy), dev(w), dev(x), 1, pad)
        dx = cnn.cnn_conv_bwd_data(ctx, dev(dy), dev(w), H, H, 1, pad)
        assert torch.equal(dz, cnn.cnn_relu_bwd(ctx, dev(x), dx))
        ref, s = oracle.conv_bwd_data(dy, w, H, H, 1, pad, with_abs=True)
        P.check_contraction("dz", P.np_(dz), np.where(x > 0, ref, 0.0), s)
    zz = synth.randn(97, 4, (3, 5, 8, 12)); zz[0, 0, :2, :2] = -1.0
    aa = cnn.cnn_relu_fwd(ctx, dev(zz)); y, arg = cnn.cnn_maxpool2_fwd(ctx, aa)
    g = dev(synth.randn(97, 5, tuple(y.shape)))
    fused = cnn.cnn_maxpool2_relu_bwd(ctx, g, arg, y, 8, 12)
    assert torch.equal(fused, cnn.cnn_relu_bwd(ctx, dev(zz), cnn.cnn_maxpool2_bwd(ctx, g, arg, 8, 12)))


def test_fused_conv_relu_pool_equals_the_unfused_sequence(cnn, ctx):
    # conv_fwd_relu_pool == maxpool2_fwd(conv_fwd_relu(x, w)), values and window positions bit for bit: the first
    # layer shape (C = 3, two wave columns), whole / sliced / ragged tiles, tiles spanning images, 5x5, odd N;
    # and against the oracle
    for (N, C, H, K, R, pad) in [(2, 3, 224, 64, 3, 1), (3, 16, 28, 72, 3, 1), (2, 64, 28, 128, 3, 1), (5, 32, 14, 48, 3, 1),
                                 (3, 128, 12, 64, 3, 1), (1, 8, 112, 136, 3, 1), (2, 8, 28, 40, 5, 0), (3, 64, 56, 128, 3, 1),
                                 (7, 8, 8, 40, 3, 1)]:
        say("fused pool case", (N, C, H, K, R, pad))
        x = synth.randn(98, 1, (N, C, H, H)); w = synth.randn(98, 2, (K, C, R, R), 0.1)
        r = cnn.cnn_conv_fwd_relu_pool(ctx, dev(x), dev(w), 1, pad)
        assert r is not None, "the tiled kernel serves these shapes"
        a, arg = r
        a2, arg2 = cnn.cnn_maxpool2_fwd(ctx, cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), 1, pad))
        torch.cuda.synchronize()
        assert torch.equal(a, a2)
        assert torch.equal(arg, arg2)
        P.check_trace_item(("conv_fwd_relu_pool", 0, 0, dev(x), dev(w), a, arg), 0, [("conv", C, K, R, R, 1, pad)], True)
        # the way back: conv_bwd_data_unpool_relu == maxpool2_relu_bwd(conv_bwd_data(dy, w), arg, a) for a layer whose
        # input is that pooled activation
        K2 = 40
        w2 = synth.randn(98, 3, (K2, K, 3, 3), 0.1)
        Hp = a.shape[2]
        dy2 = synth.randn(98, 4, (N, K2, Hp, Hp))
        dz = cnn.cnn_conv_bwd_data_unpool_relu(ctx, dev(dy2), dev(w2), arg, a, 1, 1)
        assert dz is not None
        dz2 = cnn.cnn_maxpool2_relu_bwd(ctx, cnn.cnn_conv_bwd_data(ctx, dev(dy2), dev(w2), Hp, Hp, 1, 1), arg, a, 2 * Hp, 2 * Hp)
        torch.cuda.synchronize()
        assert torch.equal(dz, dz2)
        P.check_trace_item(("conv_bwd_data_unpool_relu", 0, 0, dev(dy2), dev(w2), arg, a, dz), 0,
                           [("conv", K, K2, 3, 3, 1, 1)], True)
    # odd output sizes are refused before anything is launched
    L = cnn.lib(); z = dev(np.zeros((1, 1, 5, 5), np.float32)); b = torch.zeros(4, dtype=torch.uint8, device="cuda")
    assert L.cnn_conv_fwd_relu_pool(ctx.handle, 1, 1, 5, 5, 1, 3, 3, 1, 1, z.data_ptr(), z.data_ptr(), z.data_ptr(), b.data_ptr()) == -1


@pytest.mark.parametrize("case", [(11, 256, 20, 256), (12, 256, 20, 512)])
def test_fused_pool_where_the_two_calls_cut_the_contraction_differently(cnn, ctx, case):
    # 20 x 20 images: pooling wants tiles of whole row pairs, the plain call takes 11 rows: the two plans slice the
    # contraction differently, so the fused result equals the unfused pair only up to rounding (and the window
    # positions up to near-ties); against the oracle both hold the tolerance
    N, C, H, K = case
    say("fused pool, differently planned", case)
    x = synth.randn(81, 1, (N, C, H, H)); w = synth.randn(81, 2, (K, C, 3, 3), 0.05)
    a, arg = cnn.cnn_conv_fwd_relu_pool(ctx, dev(x), dev(w), 1, 1)
    a2, arg2 = cnn.cnn_maxpool2_fwd(ctx, cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), 1, 1))
    torch.cuda.synchronize()
    assert float((a - a2).abs().max()) <= 2e-5 * float(a2.abs().max())
    assert float((arg != arg2).float().mean()) < 1e-3
    P.check_trace_item(("conv_fwd_relu_pool", 0, 0, dev(x), dev(w), a, arg), 0, [("conv", C, K, 3, 3, 1, 1)], True)


@pytest.mark.parametrize("cfg,n", [(2, None), (5, None), (4, 8), (3, 8), (4, None), (3, None)])
def test_training_steps_with_folded_sgd_equal_the_separate_update(cnn, ctx, cfg, n):
    # two iterations (the second one uses the first one's velocity) of each workload, once with the update inside
    # the weight gradients and once as gradient arena + one cnn_sgd_update: same weights and velocity, bit for bit
    # (n = None: the workload's own minibatch -- 64 for VGG-A and OverFeat-FAST, what the benchmark times)
    from paper_1602_06709_amd.net import Net
    wl = synth.workload(cfg, n)
    if not wl.sgd:       # workloads defined without an update take one here
        wl = dataclasses.replace(wl, sgd=True, lr=0.01, momentum=0.9)
    say(f"folded-sgd steps cfg{cfg} N={wl.input_shape[0]}")
    nets = [Net(ctx, wl, synth.make_weights(wl), fuse_sgd=f) for f in (True, False)]
    for it in range(2):
        for net in nets:
            net.set_input(synth.make_input(wl), synth.make_labels(wl) if wl.loss else None)
            if not wl.loss:
                net.set_upstream(synth.make_upstream(wl))
            net.step()
        torch.cuda.synchronize()
        assert torch.equal(nets[0].w_arena, nets[1].w_arena), f"weights differ after iteration {it}"
        if nets[0].v_arena is not None:
            assert torch.equal(nets[0].v_arena, nets[1].v_arena), f"velocity differs after iteration {it}"


@pytest.mark.parametrize("case", [(28, 224), (56, 100), (40, 158), (14, 224)])
def test_first_layer_band_kernel_with_pool(cnn, ctx, case):
    # 3 -> 64 features, 3x3 / pad 1, 224 columns, conv -> ReLU -> 2x2 max-pool in one kernel that walks bands of 14
    # rows (served from 224 bands up): whole bands, a ragged last band (100 = 7 x 14 + 2; 158 = 11 x 14 + 4), all
    # elements against the oracle; the unfused sequence must agree wherever the window's maximum is not a near-tie
    N, H = case
    say("first-layer band kernel", case)
    x = synth.randn(87, 1, (N, 3, H, 224)); w = synth.randn(87, 2, (64, 3, 3, 3), 0.2)
    r = cnn.cnn_conv_fwd_relu_pool(ctx, dev(x), dev(w), 1, 1)
    assert r is not None
    a, arg = r
    torch.cuda.synchronize()
    P.check_trace_item(("conv_fwd_relu_pool", 0, 0, dev(x), dev(w), a, arg), 0, [("conv", 3, 64, 3, 3, 1, 1)], True)
    a2, arg2 = cnn.cnn_maxpool2_fwd(ctx, cnn.cnn_conv_fwd_relu(ctx, dev(x), dev(w), 1, 1))
    torch.cuda.synchronize()
    assert float((a - a2).abs().max()) <= 1e-4
    assert float((arg != arg2).float().mean()) < 1e-3


@pytest.mark.parametrize("case", [(2, 3, 224, 224, 64, 1), (3, 3, 30, 44, 40, 1), (5, 3, 18, 24, 16, 0), (2, 3, 64, 130, 64, 1),
                                  (16, 3, 224, 224, 64, 1)])
def test_first_layer_weight_gradient_from_the_pooled_gradient(cnn, ctx, case):
    # dw = conv_bwd_weight(x, maxpool2_bwd(dpool, arg)) without the full-size gradient: bit for bit what the two calls
    # give (same kernel, the gradient formed on its way into LDS), and against the oracle; plain and with the SGD
    # step folded in; then a shape the kernel does not serve is refused
    N, C, H, W, K, pad = case
    say("pooled weight gradient", case)
    P_, Q_ = H + 2 * pad - 2, W + 2 * pad - 2
    x = synth.randn(89, 1, (N, C, H, W))
    dpool = synth.randn(89, 2, (N, K, P_ // 2, Q_ // 2))
    dpool[0, 0, :2] = 0.0                                                       # a closed ReLU region
    arg = (synth.randn(89, 3, dpool.shape) * 1e3).astype(np.int64) % 4
    arg = arg.astype(np.uint8)
    assert cnn.conv_bwd_weight_unpool_serves(N, C, H, W, K, 3, 3, 1, pad)
    dw = cnn.cnn_conv_bwd_weight_unpool(ctx, dev(x), dev(dpool), dev(arg), 3, 3, 1, pad)
    assert dw is not None
    full = cnn.cnn_maxpool2_bwd(ctx, dev(dpool), dev(arg), P_, Q_)
    dw2 = cnn.cnn_conv_bwd_weight(ctx, dev(x), full, 3, 3, 1, pad)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2)
    P.check_trace_item(("conv_bwd_weight_unpool", 0, 0, dev(x), dev(dpool), dev(arg), dw), 0, [("conv", C, K, 3, 3, 1, pad)],
                       N * H * W <= 2 * 224 * 224, n_samples_wgrad=600)
    w0 = synth.randn(89, 4, (K, C, 3, 3), 0.1); v0 = synth.randn(89, 5, (K, C, 3, 3), 0.01)
    w1, v1 = dev(w0), dev(v0)
    cnn.cnn_conv_bwd_weight_unpool(ctx, dev(x), dev(dpool), dev(arg), 3, 3, 1, pad, w=w1, v=v1, lr=0.05, momentum=0.9)
    w2, v2 = dev(w0), dev(v0)
    cnn.cnn_sgd_update(ctx, w2.view(-1), dw2.view(-1), v2.view(-1), 0.05, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(w1, w2) and torch.equal(v1, v2)


def test_pooled_weight_gradient_refuses_other_shapes(cnn, ctx):
    for (N, C, H, W, K, R, st, pad) in [(2, 3, 39, 39, 8, 11, 4, 0), (2, 3, 31, 30, 16, 3, 1, 0), (2, 16, 28, 28, 32, 3, 1, 1),
                                        (2, 3, 64, 64, 96, 3, 1, 1)]:
        assert not cnn.conv_bwd_weight_unpool_serves(N, C, H, W, K, R, R, st, pad)
        P_, Q_ = (H + 2 * pad - R) // st + 1, (W + 2 * pad - R) // st + 1
        if P_ % 2 or Q_ % 2:
            continue
        x = dev(synth.randn(88, 1, (N, C, H, W))); dp = dev(synth.randn(88, 2, (N, K, P_ // 2, Q_ // 2)))
        arg = torch.zeros(dp.shape, dtype=torch.uint8, device="cuda")
        assert cnn.cnn_conv_bwd_weight_unpool(ctx, x, dp, arg, R, R, st, pad) is None


@pytest.mark.parametrize("cfg,n", [(3, 16), (5, 256)])
def test_training_stays_finite_and_the_loss_falls(cnn, ctx, cfg, n):
    # twelve steps on the one synthetic batch: what the benchmark times must be a training run, not NaNs
    from paper_1602_06709_amd.net import Net
    wl = synth.workload(cfg, n)
    net = Net(ctx, wl, synth.make_weights(wl))
    net.set_input(synth.make_input(wl), synth.make_labels(wl))
    losses = []
    for _ in range(12):
        net.step()
        losses.append(float(net.loss_per_sample.mean()))
    say("losses", cfg, losses)
    assert all(np.isfinite(losses)) and all(bool(torch.isfinite(w).all()) for w in net.w)
    assert losses[-1] < losses[0]


def _run_folded_step_and_check(cnn, ctx, cfg, full, **kw):
    """The sequence the benchmark times -- Net.step() with the SGD update inside every weight gradient, a layer's
    backpropagation issued before it -- at the workload's own minibatch, every call against the oracle.  One step
    first, so that the checked step starts from a non-zero velocity."""
    from paper_1602_06709_amd.net import Net
    wl = synth.workload(cfg)
    say(f"folded step cfg{cfg} N={wl.input_shape[0]} full={full}")
    net = Net(ctx, wl, synth.make_weights(wl), record=True)
    assert net.fuse_sgd and wl.sgd
    net.set_input(synth.make_input(wl), synth.make_labels(wl))
    net.step()
    torch.cuda.synchronize()
    w0 = [P.np_(w).copy() for w in net.w]
    v0 = [P.np_(v).copy() if v is not None else None for v in net.v]
    net.step()
    torch.cuda.synchronize()
    ops = [item[0] for item in net.trace]
    n_weighted = sum(1 for L in wl.layers if L[0] in ("conv", "fc"))
    assert sum("_sgd" in op for op in ops) == n_weighted, ops      # every update went through a folded call
    assert not any(op in ("conv_bwd_weight", "fc_bwd", "fc_bwd_act", "conv_bwd_weight_unpool") for op in ops), ops
    for item in net.trace:
        if "_sgd" not in item[0]:
            # the call read this step's weights, which the folded update has since overwritten in place
            wi = item[2] if item[0].startswith(("conv_", "fc_")) else None
            item = tuple(w0[wi] if (wi is not None and isinstance(t, torch.Tensor) and t.data_ptr() == net.w[wi].data_ptr())
                         else t for t in item)
        r = P.check_trace_item(item, cfg, wl.layers, full, pre=(w0, v0), lr=wl.lr, momentum=wl.momentum, **kw)
        say(f"  {item[0]}@{item[1]} rel-L2 {r:.2e}")


def test_config5_dnn7_n1024_full_tensors(cnn, ctx):
    _run_and_check(cnn, ctx, 5, None, True)


def test_config5_dnn7_n1024_folded_step_full_tensors(cnn, ctx):
    _run_folded_step_and_check(cnn, ctx, 5, True)


def test_config3_vgg_a_full_n64_sampled(cnn, ctx):
    _run_and_check(cnn, ctx, 3, None, False, n_samples=8000, n_samples_wgrad=400)


def test_config3_vgg_a_full_n64_folded_step_sampled(cnn, ctx):
    _run_folded_step_and_check(cnn, ctx, 3, False, n_samples=8000, n_samples_wgrad=400)


def test_config4_overfeat_fast_n64_sampled(cnn, ctx):
    _run_and_check(cnn, ctx, 4, None, False, n_samples=8000, n_samples_wgrad=400)
