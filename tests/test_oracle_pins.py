"""Pins for the CPU oracle: it is checked against things other than itself.

  * a hand-worked example (tests/golden/hand_conv.txt), closed forms and invariants;
  * library routines it does not use: torch's fp64 conv2d / autograd, scipy's correlate2d,
    numpy matmul, torch max-pool / softmax / sigmoid;
  * the trilinear-form identities tying the three passes together (Section 2.1: the three
    operations are the same loop nest), and exact finite differences;
  * the paper's printed numbers (tests/golden/paper_values.txt).
All CPU-only.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1602_06709_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


def _rand(seed, shape, lo=-1, hi=1):
    return np.random.default_rng(seed).uniform(lo, hi, shape).astype(np.float32)


CASES = [  # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 7, 4, 3, 3, 1, 1),
    (1, 2, 9, 6, 3, 3, 3, 1, 0),
    (2, 3, 8, 11, 2, 5, 5, 1, 0),
    (1, 3, 23, 19, 4, 11, 11, 4, 0),
    (2, 2, 9, 9, 3, 3, 3, 2, 1),
    (1, 4, 6, 5, 5, 1, 1, 1, 0),
    (2, 2, 10, 7, 3, 2, 3, 2, 2),   # non-square kernel, stride leaves a remainder
    (1, 1, 12, 12, 1, 5, 5, 3, 2),
]


# ---------------------------------------------------------------- hand-worked example
def test_hand_worked_example():
    g = _kv(os.path.join(GOLD, "hand_conv.txt"))
    arr = lambda k: np.array([float(v) for v in g[k].split()], np.float32)
    x = arr("x").reshape(1, 1, 3, 3); w = arr("w").reshape(1, 1, 2, 2); go = arr("g").reshape(1, 1, 2, 2)
    assert np.array_equal(oracle.conv_fwd(x, w, 1, 0).ravel(), arr("y"))
    assert np.array_equal(oracle.conv_bwd_weight(x, go, 2, 2, 1, 0).ravel(), arr("dw"))
    assert np.array_equal(oracle.conv_bwd_data(go, w, 3, 3, 1, 0).ravel(), arr("dx"))


# ---------------------------------------------------------------- closed forms
def test_all_ones_counts_valid_taps():
    C = 5
    x = np.ones((1, C, 6, 8), np.float32); w = np.ones((2, C, 3, 3), np.float32)
    y = oracle.conv_fwd(x, w, 1, 0)
    assert np.all(y == 9 * C)
    y = oracle.conv_fwd(x, w, 1, 1)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[:, :, 0, 1:-1] == 6 * C) and np.all(y[:, :, 1:-1, -1] == 6 * C)
    assert y[0, 0, 0, 0] == 4 * C and y[0, 1, -1, -1] == 4 * C


def test_delta_filter_is_identity_and_shift():
    x = _rand(1, (2, 3, 5, 6))
    w = np.zeros((3, 3, 3, 3), np.float32)
    for k in range(3):
        w[k, k, 1, 1] = 1
    assert np.array_equal(oracle.conv_fwd(x, w, 1, 1), x.astype(np.float64))
    # a tap at (r,s)=(0,2) reads x[p-1, q+1]: cross-correlation, no flip
    w = np.zeros((1, 3, 3, 3), np.float32); w[0, 1, 0, 2] = 1
    y = oracle.conv_fwd(x, w, 1, 1)
    exp = np.zeros((2, 5, 6)); exp[:, 1:, :-1] = x[:, 1, :-1, 1:]
    assert np.array_equal(y[:, 0], exp)


def test_1x1_conv_is_per_pixel_matmul():
    x = _rand(2, (2, 6, 4, 5)); w = _rand(3, (7, 6, 1, 1))
    y = oracle.conv_fwd(x, w, 1, 0)
    exp = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_allclose(y, exp, rtol=1e-14, atol=1e-14)


def test_stride_subsamples_stride1():
    x = _rand(4, (1, 2, 11, 13)); w = _rand(5, (3, 2, 3, 3))
    y1 = oracle.conv_fwd(x, w, 1, 1)
    for st in (2, 3, 4):
        ys = oracle.conv_fwd(x, w, st, 1)
        assert np.array_equal(ys, y1[:, :, ::st, ::st][:, :, :ys.shape[2], :ys.shape[3]])


def test_linearity():
    x1, x2 = _rand(6, (1, 2, 6, 6)), _rand(7, (1, 2, 6, 6)); w = _rand(8, (3, 2, 3, 3))
    a = oracle.conv_fwd(x1, w, 1, 1) + oracle.conv_fwd(x2, w, 1, 1)
    # x1 + x2 in fp32 rounds, so feed the exactly representable sum
    xs = (x1.astype(np.float64) + x2.astype(np.float64)).astype(np.float32)
    exact = np.array_equal(xs.astype(np.float64), x1.astype(np.float64) + x2.astype(np.float64))
    b = oracle.conv_fwd(xs, w, 1, 1)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-6 if not exact else 1e-13)


# ---------------------------------------------------------------- library routines
@pytest.mark.parametrize("case", CASES)
def test_conv_three_passes_vs_torch_fp64(case):
    N, C, H, W, K, R, S, st, pad = case
    x = _rand(10, (N, C, H, W)); w = _rand(11, (K, C, R, S))
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=st, padding=pad)
    g = _rand(12, tuple(yt.shape))
    yt.backward(torch.tensor(g, dtype=torch.float64))
    y, s = oracle.conv_fwd(x, w, st, pad, with_abs=True)
    assert y.shape == tuple(yt.shape)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-13, atol=1e-13)
    dx, sdx = oracle.conv_bwd_data(g, w, H, W, st, pad, with_abs=True)
    dw, sdw = oracle.conv_bwd_weight(x, g, R, S, st, pad, with_abs=True)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-13, atol=1e-13)
    # S = sum |a*b| is the same contraction on absolute values: torch's forward and its autograd
    # on |x|, |w|, |g| give the S of all three passes
    xa = torch.tensor(np.abs(x), dtype=torch.float64, requires_grad=True)
    wa = torch.tensor(np.abs(w), dtype=torch.float64, requires_grad=True)
    sa = torch.nn.functional.conv2d(xa, wa, stride=st, padding=pad)
    sa.backward(torch.tensor(np.abs(g), dtype=torch.float64))
    np.testing.assert_allclose(s, sa.detach().numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sdx, xa.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sdw, wa.grad.numpy(), rtol=1e-13, atol=1e-13)
    # the sampled forms return the same (value, S) pairs, pinned here against torch directly
    for (v, sv), ref, sref in (
            (oracle.conv_fwd_at(x, w, np.arange(y.size), st, pad), yt.detach().numpy(), sa.detach().numpy()),
            (oracle.conv_bwd_data_at(g, w, H, W, np.arange(dx.size), st, pad), xt.grad.numpy(), xa.grad.numpy()),
            (oracle.conv_bwd_weight_at(x, g, R, S, np.arange(dw.size), st, pad), wt.grad.numpy(), wa.grad.numpy())):
        np.testing.assert_allclose(v, ref.ravel(), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(sv, sref.ravel(), rtol=1e-13, atol=1e-13)


def test_conv_vs_scipy_correlate2d():
    from scipy.signal import correlate2d
    x = _rand(20, (1, 3, 9, 8)); w = _rand(21, (2, 3, 3, 3))
    y = oracle.conv_fwd(x, w, 1, 1)
    for k in range(2):
        exp = sum(correlate2d(np.pad(x[0, c].astype(np.float64), 1), w[k, c].astype(np.float64), mode="valid")
                  for c in range(3))
        np.testing.assert_allclose(y[0, k], exp, rtol=1e-13, atol=1e-13)


def test_bwd_data_is_fwd_with_rotated_swapped_filter():
    # textbook identity for stride 1: dx = conv_fwd(dy, rot180(w) with C/K swapped, pad R-1-pad)
    x_shape = (2, 3, 7, 6); w = _rand(22, (4, 3, 3, 3)); g = _rand(23, (2, 4, 7, 6))
    dx = oracle.conv_bwd_data(g, w, 7, 6, 1, 1)
    wr = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    np.testing.assert_allclose(dx, oracle.conv_fwd(g, wr, 1, 1), rtol=1e-13, atol=1e-13)
    assert dx.shape == x_shape


# ---------------------------------------------------------------- trilinear identities
@pytest.mark.parametrize("case", CASES + [(2, 3, 32, 32, 16, 3, 3, 1, 1)])
def test_adjoint_identities(case):
    N, C, H, W, K, R, S, st, pad = case
    x = _rand(30, (N, C, H, W)); w = _rand(31, (K, C, R, S))
    y = oracle.conv_fwd(x, w, st, pad)
    g = _rand(32, y.shape)
    t = np.sum(y * g)
    t_x = np.sum(x.astype(np.float64) * oracle.conv_bwd_data(g, w, H, W, st, pad))
    t_w = np.sum(w.astype(np.float64) * oracle.conv_bwd_weight(x, g, R, S, st, pad))
    scale = np.sum(np.abs(y * g)) + 1e-30
    assert abs(t - t_x) / scale < 1e-12 and abs(t - t_w) / scale < 1e-12


def test_finite_differences_are_exact_for_a_trilinear_form():
    # T(x,w,g) = <conv_fwd(x,w), g> is linear in w and in x: a unit step gives the derivative exactly.
    N, C, H, W, K, R, S, st, pad = 1, 2, 5, 4, 2, 3, 3, 1, 1
    x = np.round(_rand(40, (N, C, H, W)) * 8).astype(np.float32)        # small integers: exact arithmetic
    w = np.round(_rand(41, (K, C, R, S)) * 8).astype(np.float32)
    g = np.round(_rand(42, (N, K, H, W)) * 8).astype(np.float32)
    T = lambda xx, ww: np.sum(oracle.conv_fwd(xx, ww, st, pad) * g)
    dw = oracle.conv_bwd_weight(x, g, R, S, st, pad); dx = oracle.conv_bwd_data(g, w, H, W, st, pad)
    t0 = T(x, w)
    for idx in np.ndindex(*w.shape):
        w2 = w.copy(); w2[idx] += 1
        assert T(x, w2) - t0 == dw[idx]
    for idx in np.ndindex(*x.shape):
        x2 = x.copy(); x2[idx] += 1
        assert T(x2, w) - t0 == dx[idx]


# ---------------------------------------------------------------- sampled forms vs full forms
@pytest.mark.parametrize("case", CASES)
def test_sampled_forms_match_full_forms(case):
    N, C, H, W, K, R, S, st, pad = case
    x = _rand(50, (N, C, H, W)); w = _rand(51, (K, C, R, S))
    y, sy = oracle.conv_fwd(x, w, st, pad, with_abs=True)
    g = _rand(52, y.shape)
    dx, sx = oracle.conv_bwd_data(g, w, H, W, st, pad, with_abs=True)
    dw, sw = oracle.conv_bwd_weight(x, g, R, S, st, pad, with_abs=True)
    for full, sfull, fn in ((y, sy, lambda i: oracle.conv_fwd_at(x, w, i, st, pad)),
                            (dx, sx, lambda i: oracle.conv_bwd_data_at(g, w, H, W, i, st, pad)),
                            (dw, sw, lambda i: oracle.conv_bwd_weight_at(x, g, R, S, i, st, pad))):
        idx = np.arange(full.size)
        v, s = fn(idx)
        np.testing.assert_allclose(v, full.ravel(), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(s, sfull.ravel(), rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- fully-connected
def test_fc_is_matmul_and_is_the_1x1_special_case():
    N, I, O = 5, 37, 11
    x = _rand(60, (N, I)); w = _rand(61, (O, I)); g = _rand(62, (N, O))
    x64, w64, g64 = x.astype(np.float64), w.astype(np.float64), g.astype(np.float64)
    y, s = oracle.fc_fwd(x, w, with_abs=True)
    np.testing.assert_allclose(y, x64 @ w64.T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(s, np.abs(x64) @ np.abs(w64).T, rtol=1e-13, atol=1e-13)
    dx, sdx = oracle.fc_bwd_data(g, w, with_abs=True)
    dw, sdw = oracle.fc_bwd_weight(x, g, with_abs=True)
    np.testing.assert_allclose(dx, g64 @ w64, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dw, g64.T @ x64, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sdx, np.abs(g64) @ np.abs(w64), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sdw, np.abs(g64).T @ np.abs(x64), rtol=1e-13, atol=1e-13)
    # Section 2.1: FC is the conv loop nest with k_h = k_w = out_h = out_w = 1
    yc = oracle.conv_fwd(x.reshape(N, I, 1, 1), w.reshape(O, I, 1, 1), 1, 0)
    np.testing.assert_allclose(yc.reshape(N, O), y, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(oracle.conv_bwd_weight(x.reshape(N, I, 1, 1), g.reshape(N, O, 1, 1), 1, 1, 1, 0)
                               .reshape(O, I), oracle.fc_bwd_weight(x, g), rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(oracle.conv_bwd_data(g.reshape(N, O, 1, 1), w.reshape(O, I, 1, 1), 1, 1, 1, 0)
                               .reshape(N, I), oracle.fc_bwd_data(g, w), rtol=1e-14, atol=1e-14)
    # sampled forms: value and S against numpy matmul (not against the full forms)
    for ref, sref, fn in ((x64 @ w64.T, np.abs(x64) @ np.abs(w64).T, lambda i: oracle.fc_fwd_at(x, w, i)),
                          (g64 @ w64, np.abs(g64) @ np.abs(w64), lambda i: oracle.fc_bwd_data_at(g, w, i)),
                          (g64.T @ x64, np.abs(g64).T @ np.abs(x64), lambda i: oracle.fc_bwd_weight_at(x, g, i))):
        v, sv = fn(np.arange(ref.size))
        np.testing.assert_allclose(v, ref.ravel(), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(sv, sref.ravel(), rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- SGD
def test_sgd_closed_form_constant_gradient():
    n, lr, mu, steps = 17, 0.01, 0.9, 12
    w0 = _rand(70, n); g = _rand(71, n)
    w = w0.astype(np.float64); v = np.zeros(n)
    for _ in range(steps):
        # the oracle takes fp32-valued inputs: feed exactly representable states
        w32, v32 = w.astype(np.float32), v.astype(np.float32)
        wn, vn = oracle.sgd_update(w32, g, v32, lr, mu)
        np.testing.assert_allclose(vn, mu * v32.astype(np.float64) + g, rtol=1e-15)
        w, v = wn, vn
    # closed form in exact arithmetic: w_t = w0 - lr*g*sum_{j<t} (1-mu^(j+1))/(1-mu)
    coef = sum((1 - mu ** (j + 1)) / (1 - mu) for j in range(steps))
    np.testing.assert_allclose(w, w0 - lr * g.astype(np.float64) * coef, rtol=0, atol=5e-6)
    # mu = 0, no velocity buffer: w - lr*g
    wn, vn = oracle.sgd_update(w0, g, None, lr, 0.0)
    assert vn is None
    np.testing.assert_allclose(wn, w0.astype(np.float64) - lr * g.astype(np.float64), rtol=1e-15)
    # sign: a positive gradient lowers the weight
    assert oracle.sgd_update(np.ones(1, np.float32), np.ones(1, np.float32), None, 0.5, 0.0)[0][0] == 0.5


# ---------------------------------------------------------------- layouts (Section 2.3)
@pytest.mark.parametrize("sw", [4, 8, 16])
def test_blocked_layouts_are_the_stated_permutations(sw):
    N, C, H, W, K, R, S = 2, 11, 3, 5, 13, 3, 2
    x = _rand(80, (N, C, H, W)); w = _rand(81, (K, C, R, S))
    CB, KB = -(-C // sw), -(-K // sw)
    xp = np.zeros((N, CB * sw, H, W), np.float32); xp[:, :C] = x
    exp = xp.reshape(N, CB, sw, H, W).transpose(0, 1, 3, 4, 2)          # N x C/SW x H x W x SW
    got = oracle.pack_act(x, sw)
    assert np.array_equal(got, exp)
    assert np.array_equal(oracle.unpack_act(got, C), x)
    # weights: IFM x OFM/SW x KH x KW x SW (lanes over output features)
    wp = np.zeros((KB * sw, C, R, S), np.float32); wp[:K] = w
    exp = wp.reshape(KB, sw, C, R, S).transpose(2, 0, 3, 4, 1)
    got = oracle.pack_wt(w, sw, transpose=False)
    assert np.array_equal(got, exp)
    assert np.array_equal(oracle.unpack_wt(got, K, C, False), w)
    # transpose-weights: OFM x IFM/SW x KH x KW x SW (lanes over input features)
    wp = np.zeros((K, CB * sw, R, S), np.float32); wp[:, :C] = w
    exp = wp.reshape(K, CB, sw, R, S).transpose(0, 1, 3, 4, 2)
    got = oracle.pack_wt(w, sw, transpose=True)
    assert np.array_equal(got, exp)
    assert np.array_equal(oracle.unpack_wt(got, K, C, True), w)


# ---------------------------------------------------------------- glue ops
def test_relu_pool_sigmoid_softmax_vs_torch():
    z = _rand(90, (2, 3, 6, 8), -2, 2)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    a = torch.relu(zt); da = _rand(91, z.shape)
    a.backward(torch.tensor(da, dtype=torch.float64))
    assert np.array_equal(oracle.relu_fwd(z), a.detach().numpy())
    assert np.array_equal(oracle.relu_bwd(z, da), zt.grad.numpy())
    assert oracle.relu_bwd(np.zeros(1, np.float32), np.ones(1, np.float32))[0] == 0      # ReLU'(0) = 0

    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.max_pool2d(zt, 2, 2); dy = _rand(92, tuple(y.shape))
    y.backward(torch.tensor(dy, dtype=torch.float64))
    yo, arg = oracle.maxpool2_fwd(z)
    assert np.array_equal(yo, y.detach().numpy())
    dxo = oracle.maxpool2_bwd(dy, arg, 6, 8)
    assert np.array_equal(dxo, zt.grad.numpy())
    assert abs(dxo.sum() - dy.astype(np.float64).sum()) < 1e-12                            # conserves the gradient
    # ties: the first maximum in row-major window order takes the gradient
    tie = np.zeros((1, 1, 2, 2), np.float32)
    _, arg = oracle.maxpool2_fwd(tie)
    assert arg.ravel()[0] == 0
    tie[0, 0, 0, 1] = tie[0, 0, 1, 0] = 3
    assert oracle.maxpool2_fwd(tie)[1].ravel()[0] == 1

    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    s = torch.sigmoid(zt); s.backward(torch.tensor(da, dtype=torch.float64))
    so = oracle.sigmoid_fwd(z)
    np.testing.assert_allclose(so, s.detach().numpy(), rtol=1e-14)
    np.testing.assert_allclose(oracle.sigmoid_bwd(so.astype(np.float32), da),
                               da.astype(np.float64) * so.astype(np.float32).astype(np.float64)
                               * (1 - so.astype(np.float32).astype(np.float64)), rtol=1e-14)
    np.testing.assert_allclose(oracle.sigmoid_bwd(so.astype(np.float32), da), zt.grad.numpy(), rtol=1e-6, atol=1e-8)

    N, O = 6, 19
    lg = _rand(93, (N, O), -5, 5); lab = np.random.default_rng(94).integers(0, O, N).astype(np.int32)
    lt = torch.tensor(lg, dtype=torch.float64, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(lt, torch.tensor(lab, dtype=torch.long), reduction="mean")
    loss.backward()
    lo, dz = oracle.softmax_xent(lg, lab)
    assert abs(lo - loss.item()) < 1e-13
    np.testing.assert_allclose(dz, lt.grad.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    # large logits do not overflow (max-subtraction form)
    big = np.array([[1000.0, 0.0, -1000.0]], np.float32)
    lo, dz = oracle.softmax_xent(big, np.array([0], np.int32))
    assert np.isfinite(lo) and lo < 1e-12 and np.all(np.isfinite(dz))


# ---------------------------------------------------------------- FLOP counter and the paper's numbers
def _net_macs(layers, input_shape):
    """MACs per image of the conv and fc layers, from shapes alone (no oracle call)."""
    wl = synth.Workload(0, "x", layers, input_shape, False)
    shp = [tuple(input_shape)] + synth.shapes(wl)
    conv = fc = 0
    for L, s_out in zip(layers, shp[1:]):
        if L[0] == "conv":
            conv += L[1] * L[2] * L[3] * L[4] * s_out[2] * s_out[3]
        elif L[0] == "fc":
            fc += L[1] * L[2]
    return conv, fc


def test_flop_counter_and_printed_numbers():
    g = {k: float(v) for k, v in _kv(os.path.join(GOLD, "paper_values.txt")).items()}
    # Section 3.1 formula by hand for the small single-layer workload: 2*2*16*32*32*27
    assert oracle.conv_flops_per_pass(2, 3, 32, 32, 16, 3, 3, 1, 1) == 1769472
    assert oracle.conv_flops_per_pass(1, 3, 231, 231, 96, 11, 11, 4, 0) == 2 * 3 * 96 * 121 * 56 * 56
    assert oracle.fc_flops_per_pass(64, 25088, 4096) == 2 * 64 * 25088 * 4096
    # VGG-A: the layer list gives 7.609 GMAC per image; the footnote's 33.6 GFlops lies between the
    # two-pass and three-pass totals of the paper's own formula (it matches neither exactly).
    conv, fc = _net_macs(synth.VGG_A_CONV + synth.VGG_A_FC, (1, 3, 224, 224))
    total = sum(oracle.conv_flops_per_pass(1, L[1], h, h, L[2], 3, 3, 1, 1)
                for L, h in zip([l for l in synth.VGG_A_CONV if l[0] == "conv"],
                                [224, 112, 56, 56, 28, 28, 14, 14]))
    assert total == g["flops_per_mac"] * conv
    fwd = g["flops_per_mac"] * (conv + fc) / 1e9
    assert abs(fwd - 15.218) < 0.005
    assert 2 * fwd < g["vgg_a_gflops_per_image"] < g["comp_passes"] * fwd
    # parameter counts (no biases anywhere in the paper's loops)
    assert sum(int(np.prod(s)) for s in synth.weight_shapes(synth.workload(3))) == 132851392
    assert sum(int(np.prod(s)) for s in synth.weight_shapes(synth.workload(4))) == 145909792
    # CD-DNN: 3 passes x 2 FLOP/MAC x 40.9 M MAC per frame at 4600 frames/s on a 1.7 TFLOP/s peak
    # is 66 %, in line with the ~70 % the paper states for fully-connected layers.
    _, fc = _net_macs(synth.DNN7, (1, 440))
    assert fc == 40927232
    eff = g["comp_passes"] * g["flops_per_mac"] * fc * g["cddnn_frames_per_s"] / (g["cddnn_peak_tflops"] * 1e12)
    assert abs(eff - g["fc_efficiency"]) < 0.06
    # Section 2.2 bytes-per-FLOP of the unblocked loop: pins in_h = out_h*s + k_h - 1 (12x12 out, 3x3)
    bf = 4 * (12 * 12 + 14 * 14 + 9) / (2 * 9 * 12 * 12)
    assert abs(bf - g["bf_unblocked_c5"]) < 0.005
    assert oracle.out_dim(14, 3, 1, 0) == 12 and oracle.out_dim(12, 3, 1, 1) == 12
    assert oracle.out_dim(231, 11, 4, 0) == 56 and oracle.out_dim(28, 5, 1, 0) == 24


def test_workload_shapes():
    s = synth.shapes(synth.workload(2))
    assert s[0] == (4, 64, 224, 224) and s[-1] == (4, 512, 7, 7)
    s = synth.shapes(synth.workload(4))
    assert s[0] == (64, 96, 56, 56) and s[-1] == (64, 1000)
    assert (64, 36864) in s
    s = synth.shapes(synth.workload(5))
    assert s[-1] == (1024, 9304)
    assert synth.shapes(synth.workload(3))[-1] == (64, 1000)
